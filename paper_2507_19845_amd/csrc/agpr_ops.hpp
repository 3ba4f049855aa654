// Accessors for hand-placed accumulators in AGPRs: register numbers must appear literally
// in the instruction text, so there is one specialisation per register (range).  Mechanical.
#pragma once
#include "common.hpp"

namespace gpts {

typedef int i32x4_t __attribute__((ext_vector_type(4)));

// a[R:R+3] += X (16 x 32) * Y (32 x 16), bf16 operands, R a multiple of 4
template <int R> __device__ __forceinline__ void mfma16_at(const bf16x8& x, const bf16x8& y);
// value of AGPR R (after the matrix pipeline has drained)
template <int R> __device__ __forceinline__ float agpr_read();

template <> __device__ __forceinline__ void mfma16_at<0>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[0:3], %0, %1, a[0:3]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a0", "a1", "a2", "a3"); }
template <> __device__ __forceinline__ void mfma16_at<4>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[4:7], %0, %1, a[4:7]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a4", "a5", "a6", "a7"); }
template <> __device__ __forceinline__ void mfma16_at<8>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[8:11], %0, %1, a[8:11]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a8", "a9", "a10", "a11"); }
template <> __device__ __forceinline__ void mfma16_at<12>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[12:15], %0, %1, a[12:15]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a12", "a13", "a14", "a15"); }
template <> __device__ __forceinline__ void mfma16_at<16>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[16:19], %0, %1, a[16:19]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a16", "a17", "a18", "a19"); }
template <> __device__ __forceinline__ void mfma16_at<20>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[20:23], %0, %1, a[20:23]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a20", "a21", "a22", "a23"); }
template <> __device__ __forceinline__ void mfma16_at<24>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[24:27], %0, %1, a[24:27]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a24", "a25", "a26", "a27"); }
template <> __device__ __forceinline__ void mfma16_at<28>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[28:31], %0, %1, a[28:31]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a28", "a29", "a30", "a31"); }
template <> __device__ __forceinline__ void mfma16_at<32>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[32:35], %0, %1, a[32:35]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a32", "a33", "a34", "a35"); }
template <> __device__ __forceinline__ void mfma16_at<36>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[36:39], %0, %1, a[36:39]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a36", "a37", "a38", "a39"); }
template <> __device__ __forceinline__ void mfma16_at<40>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[40:43], %0, %1, a[40:43]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a40", "a41", "a42", "a43"); }
template <> __device__ __forceinline__ void mfma16_at<44>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[44:47], %0, %1, a[44:47]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a44", "a45", "a46", "a47"); }
template <> __device__ __forceinline__ void mfma16_at<48>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[48:51], %0, %1, a[48:51]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a48", "a49", "a50", "a51"); }
template <> __device__ __forceinline__ void mfma16_at<52>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[52:55], %0, %1, a[52:55]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a52", "a53", "a54", "a55"); }
template <> __device__ __forceinline__ void mfma16_at<56>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[56:59], %0, %1, a[56:59]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a56", "a57", "a58", "a59"); }
template <> __device__ __forceinline__ void mfma16_at<60>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[60:63], %0, %1, a[60:63]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a60", "a61", "a62", "a63"); }
template <> __device__ __forceinline__ void mfma16_at<64>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[64:67], %0, %1, a[64:67]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a64", "a65", "a66", "a67"); }
template <> __device__ __forceinline__ void mfma16_at<68>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[68:71], %0, %1, a[68:71]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a68", "a69", "a70", "a71"); }
template <> __device__ __forceinline__ void mfma16_at<72>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[72:75], %0, %1, a[72:75]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a72", "a73", "a74", "a75"); }
template <> __device__ __forceinline__ void mfma16_at<76>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[76:79], %0, %1, a[76:79]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a76", "a77", "a78", "a79"); }
template <> __device__ __forceinline__ void mfma16_at<80>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[80:83], %0, %1, a[80:83]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a80", "a81", "a82", "a83"); }
template <> __device__ __forceinline__ void mfma16_at<84>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[84:87], %0, %1, a[84:87]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a84", "a85", "a86", "a87"); }
template <> __device__ __forceinline__ void mfma16_at<88>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[88:91], %0, %1, a[88:91]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a88", "a89", "a90", "a91"); }
template <> __device__ __forceinline__ void mfma16_at<92>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[92:95], %0, %1, a[92:95]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a92", "a93", "a94", "a95"); }
template <> __device__ __forceinline__ void mfma16_at<96>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[96:99], %0, %1, a[96:99]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a96", "a97", "a98", "a99"); }
template <> __device__ __forceinline__ void mfma16_at<100>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[100:103], %0, %1, a[100:103]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a100", "a101", "a102", "a103"); }
template <> __device__ __forceinline__ void mfma16_at<104>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[104:107], %0, %1, a[104:107]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a104", "a105", "a106", "a107"); }
template <> __device__ __forceinline__ void mfma16_at<108>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[108:111], %0, %1, a[108:111]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a108", "a109", "a110", "a111"); }
template <> __device__ __forceinline__ void mfma16_at<112>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[112:115], %0, %1, a[112:115]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a112", "a113", "a114", "a115"); }
template <> __device__ __forceinline__ void mfma16_at<116>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[116:119], %0, %1, a[116:119]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a116", "a117", "a118", "a119"); }
template <> __device__ __forceinline__ void mfma16_at<120>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[120:123], %0, %1, a[120:123]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a120", "a121", "a122", "a123"); }
template <> __device__ __forceinline__ void mfma16_at<124>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[124:127], %0, %1, a[124:127]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a124", "a125", "a126", "a127"); }
template <> __device__ __forceinline__ void mfma16_at<128>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[128:131], %0, %1, a[128:131]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a128", "a129", "a130", "a131"); }
template <> __device__ __forceinline__ void mfma16_at<132>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[132:135], %0, %1, a[132:135]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a132", "a133", "a134", "a135"); }
template <> __device__ __forceinline__ void mfma16_at<136>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[136:139], %0, %1, a[136:139]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a136", "a137", "a138", "a139"); }
template <> __device__ __forceinline__ void mfma16_at<140>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[140:143], %0, %1, a[140:143]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a140", "a141", "a142", "a143"); }
template <> __device__ __forceinline__ void mfma16_at<144>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[144:147], %0, %1, a[144:147]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a144", "a145", "a146", "a147"); }
template <> __device__ __forceinline__ void mfma16_at<148>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[148:151], %0, %1, a[148:151]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a148", "a149", "a150", "a151"); }
template <> __device__ __forceinline__ void mfma16_at<152>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[152:155], %0, %1, a[152:155]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a152", "a153", "a154", "a155"); }
template <> __device__ __forceinline__ void mfma16_at<156>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[156:159], %0, %1, a[156:159]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a156", "a157", "a158", "a159"); }
template <> __device__ __forceinline__ void mfma16_at<160>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[160:163], %0, %1, a[160:163]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a160", "a161", "a162", "a163"); }
template <> __device__ __forceinline__ void mfma16_at<164>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[164:167], %0, %1, a[164:167]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a164", "a165", "a166", "a167"); }
template <> __device__ __forceinline__ void mfma16_at<168>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[168:171], %0, %1, a[168:171]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a168", "a169", "a170", "a171"); }
template <> __device__ __forceinline__ void mfma16_at<172>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[172:175], %0, %1, a[172:175]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a172", "a173", "a174", "a175"); }
template <> __device__ __forceinline__ void mfma16_at<176>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[176:179], %0, %1, a[176:179]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a176", "a177", "a178", "a179"); }
template <> __device__ __forceinline__ void mfma16_at<180>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[180:183], %0, %1, a[180:183]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a180", "a181", "a182", "a183"); }
template <> __device__ __forceinline__ void mfma16_at<184>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[184:187], %0, %1, a[184:187]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a184", "a185", "a186", "a187"); }
template <> __device__ __forceinline__ void mfma16_at<188>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[188:191], %0, %1, a[188:191]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a188", "a189", "a190", "a191"); }
template <> __device__ __forceinline__ void mfma16_at<192>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[192:195], %0, %1, a[192:195]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a192", "a193", "a194", "a195"); }
template <> __device__ __forceinline__ void mfma16_at<196>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[196:199], %0, %1, a[196:199]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a196", "a197", "a198", "a199"); }
template <> __device__ __forceinline__ void mfma16_at<200>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[200:203], %0, %1, a[200:203]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a200", "a201", "a202", "a203"); }
template <> __device__ __forceinline__ void mfma16_at<204>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[204:207], %0, %1, a[204:207]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a204", "a205", "a206", "a207"); }
template <> __device__ __forceinline__ void mfma16_at<208>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[208:211], %0, %1, a[208:211]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a208", "a209", "a210", "a211"); }
template <> __device__ __forceinline__ void mfma16_at<212>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[212:215], %0, %1, a[212:215]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a212", "a213", "a214", "a215"); }
template <> __device__ __forceinline__ void mfma16_at<216>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[216:219], %0, %1, a[216:219]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a216", "a217", "a218", "a219"); }
template <> __device__ __forceinline__ void mfma16_at<220>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[220:223], %0, %1, a[220:223]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a220", "a221", "a222", "a223"); }
template <> __device__ __forceinline__ void mfma16_at<224>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[224:227], %0, %1, a[224:227]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a224", "a225", "a226", "a227"); }
template <> __device__ __forceinline__ void mfma16_at<228>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[228:231], %0, %1, a[228:231]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a228", "a229", "a230", "a231"); }
template <> __device__ __forceinline__ void mfma16_at<232>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[232:235], %0, %1, a[232:235]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a232", "a233", "a234", "a235"); }
template <> __device__ __forceinline__ void mfma16_at<236>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[236:239], %0, %1, a[236:239]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a236", "a237", "a238", "a239"); }
template <> __device__ __forceinline__ void mfma16_at<240>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[240:243], %0, %1, a[240:243]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a240", "a241", "a242", "a243"); }
template <> __device__ __forceinline__ void mfma16_at<244>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[244:247], %0, %1, a[244:247]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a244", "a245", "a246", "a247"); }
template <> __device__ __forceinline__ void mfma16_at<248>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[248:251], %0, %1, a[248:251]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a248", "a249", "a250", "a251"); }
template <> __device__ __forceinline__ void mfma16_at<252>(const bf16x8& x, const bf16x8& y) { asm volatile("v_mfma_f32_16x16x32_bf16 a[252:255], %0, %1, a[252:255]" ::"v"(__builtin_bit_cast(i32x4_t, x)), "v"(__builtin_bit_cast(i32x4_t, y)) : "a252", "a253", "a254", "a255"); }

template <> __device__ __forceinline__ float agpr_read<0>() { float v; asm volatile("v_accvgpr_read_b32 %0, a0" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<1>() { float v; asm volatile("v_accvgpr_read_b32 %0, a1" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<2>() { float v; asm volatile("v_accvgpr_read_b32 %0, a2" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<3>() { float v; asm volatile("v_accvgpr_read_b32 %0, a3" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<4>() { float v; asm volatile("v_accvgpr_read_b32 %0, a4" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<5>() { float v; asm volatile("v_accvgpr_read_b32 %0, a5" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<6>() { float v; asm volatile("v_accvgpr_read_b32 %0, a6" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<7>() { float v; asm volatile("v_accvgpr_read_b32 %0, a7" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<8>() { float v; asm volatile("v_accvgpr_read_b32 %0, a8" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<9>() { float v; asm volatile("v_accvgpr_read_b32 %0, a9" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<10>() { float v; asm volatile("v_accvgpr_read_b32 %0, a10" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<11>() { float v; asm volatile("v_accvgpr_read_b32 %0, a11" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<12>() { float v; asm volatile("v_accvgpr_read_b32 %0, a12" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<13>() { float v; asm volatile("v_accvgpr_read_b32 %0, a13" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<14>() { float v; asm volatile("v_accvgpr_read_b32 %0, a14" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<15>() { float v; asm volatile("v_accvgpr_read_b32 %0, a15" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<16>() { float v; asm volatile("v_accvgpr_read_b32 %0, a16" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<17>() { float v; asm volatile("v_accvgpr_read_b32 %0, a17" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<18>() { float v; asm volatile("v_accvgpr_read_b32 %0, a18" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<19>() { float v; asm volatile("v_accvgpr_read_b32 %0, a19" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<20>() { float v; asm volatile("v_accvgpr_read_b32 %0, a20" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<21>() { float v; asm volatile("v_accvgpr_read_b32 %0, a21" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<22>() { float v; asm volatile("v_accvgpr_read_b32 %0, a22" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<23>() { float v; asm volatile("v_accvgpr_read_b32 %0, a23" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<24>() { float v; asm volatile("v_accvgpr_read_b32 %0, a24" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<25>() { float v; asm volatile("v_accvgpr_read_b32 %0, a25" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<26>() { float v; asm volatile("v_accvgpr_read_b32 %0, a26" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<27>() { float v; asm volatile("v_accvgpr_read_b32 %0, a27" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<28>() { float v; asm volatile("v_accvgpr_read_b32 %0, a28" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<29>() { float v; asm volatile("v_accvgpr_read_b32 %0, a29" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<30>() { float v; asm volatile("v_accvgpr_read_b32 %0, a30" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<31>() { float v; asm volatile("v_accvgpr_read_b32 %0, a31" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<32>() { float v; asm volatile("v_accvgpr_read_b32 %0, a32" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<33>() { float v; asm volatile("v_accvgpr_read_b32 %0, a33" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<34>() { float v; asm volatile("v_accvgpr_read_b32 %0, a34" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<35>() { float v; asm volatile("v_accvgpr_read_b32 %0, a35" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<36>() { float v; asm volatile("v_accvgpr_read_b32 %0, a36" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<37>() { float v; asm volatile("v_accvgpr_read_b32 %0, a37" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<38>() { float v; asm volatile("v_accvgpr_read_b32 %0, a38" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<39>() { float v; asm volatile("v_accvgpr_read_b32 %0, a39" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<40>() { float v; asm volatile("v_accvgpr_read_b32 %0, a40" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<41>() { float v; asm volatile("v_accvgpr_read_b32 %0, a41" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<42>() { float v; asm volatile("v_accvgpr_read_b32 %0, a42" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<43>() { float v; asm volatile("v_accvgpr_read_b32 %0, a43" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<44>() { float v; asm volatile("v_accvgpr_read_b32 %0, a44" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<45>() { float v; asm volatile("v_accvgpr_read_b32 %0, a45" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<46>() { float v; asm volatile("v_accvgpr_read_b32 %0, a46" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<47>() { float v; asm volatile("v_accvgpr_read_b32 %0, a47" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<48>() { float v; asm volatile("v_accvgpr_read_b32 %0, a48" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<49>() { float v; asm volatile("v_accvgpr_read_b32 %0, a49" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<50>() { float v; asm volatile("v_accvgpr_read_b32 %0, a50" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<51>() { float v; asm volatile("v_accvgpr_read_b32 %0, a51" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<52>() { float v; asm volatile("v_accvgpr_read_b32 %0, a52" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<53>() { float v; asm volatile("v_accvgpr_read_b32 %0, a53" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<54>() { float v; asm volatile("v_accvgpr_read_b32 %0, a54" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<55>() { float v; asm volatile("v_accvgpr_read_b32 %0, a55" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<56>() { float v; asm volatile("v_accvgpr_read_b32 %0, a56" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<57>() { float v; asm volatile("v_accvgpr_read_b32 %0, a57" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<58>() { float v; asm volatile("v_accvgpr_read_b32 %0, a58" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<59>() { float v; asm volatile("v_accvgpr_read_b32 %0, a59" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<60>() { float v; asm volatile("v_accvgpr_read_b32 %0, a60" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<61>() { float v; asm volatile("v_accvgpr_read_b32 %0, a61" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<62>() { float v; asm volatile("v_accvgpr_read_b32 %0, a62" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<63>() { float v; asm volatile("v_accvgpr_read_b32 %0, a63" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<64>() { float v; asm volatile("v_accvgpr_read_b32 %0, a64" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<65>() { float v; asm volatile("v_accvgpr_read_b32 %0, a65" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<66>() { float v; asm volatile("v_accvgpr_read_b32 %0, a66" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<67>() { float v; asm volatile("v_accvgpr_read_b32 %0, a67" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<68>() { float v; asm volatile("v_accvgpr_read_b32 %0, a68" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<69>() { float v; asm volatile("v_accvgpr_read_b32 %0, a69" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<70>() { float v; asm volatile("v_accvgpr_read_b32 %0, a70" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<71>() { float v; asm volatile("v_accvgpr_read_b32 %0, a71" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<72>() { float v; asm volatile("v_accvgpr_read_b32 %0, a72" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<73>() { float v; asm volatile("v_accvgpr_read_b32 %0, a73" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<74>() { float v; asm volatile("v_accvgpr_read_b32 %0, a74" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<75>() { float v; asm volatile("v_accvgpr_read_b32 %0, a75" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<76>() { float v; asm volatile("v_accvgpr_read_b32 %0, a76" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<77>() { float v; asm volatile("v_accvgpr_read_b32 %0, a77" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<78>() { float v; asm volatile("v_accvgpr_read_b32 %0, a78" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<79>() { float v; asm volatile("v_accvgpr_read_b32 %0, a79" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<80>() { float v; asm volatile("v_accvgpr_read_b32 %0, a80" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<81>() { float v; asm volatile("v_accvgpr_read_b32 %0, a81" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<82>() { float v; asm volatile("v_accvgpr_read_b32 %0, a82" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<83>() { float v; asm volatile("v_accvgpr_read_b32 %0, a83" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<84>() { float v; asm volatile("v_accvgpr_read_b32 %0, a84" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<85>() { float v; asm volatile("v_accvgpr_read_b32 %0, a85" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<86>() { float v; asm volatile("v_accvgpr_read_b32 %0, a86" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<87>() { float v; asm volatile("v_accvgpr_read_b32 %0, a87" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<88>() { float v; asm volatile("v_accvgpr_read_b32 %0, a88" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<89>() { float v; asm volatile("v_accvgpr_read_b32 %0, a89" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<90>() { float v; asm volatile("v_accvgpr_read_b32 %0, a90" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<91>() { float v; asm volatile("v_accvgpr_read_b32 %0, a91" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<92>() { float v; asm volatile("v_accvgpr_read_b32 %0, a92" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<93>() { float v; asm volatile("v_accvgpr_read_b32 %0, a93" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<94>() { float v; asm volatile("v_accvgpr_read_b32 %0, a94" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<95>() { float v; asm volatile("v_accvgpr_read_b32 %0, a95" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<96>() { float v; asm volatile("v_accvgpr_read_b32 %0, a96" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<97>() { float v; asm volatile("v_accvgpr_read_b32 %0, a97" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<98>() { float v; asm volatile("v_accvgpr_read_b32 %0, a98" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<99>() { float v; asm volatile("v_accvgpr_read_b32 %0, a99" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<100>() { float v; asm volatile("v_accvgpr_read_b32 %0, a100" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<101>() { float v; asm volatile("v_accvgpr_read_b32 %0, a101" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<102>() { float v; asm volatile("v_accvgpr_read_b32 %0, a102" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<103>() { float v; asm volatile("v_accvgpr_read_b32 %0, a103" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<104>() { float v; asm volatile("v_accvgpr_read_b32 %0, a104" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<105>() { float v; asm volatile("v_accvgpr_read_b32 %0, a105" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<106>() { float v; asm volatile("v_accvgpr_read_b32 %0, a106" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<107>() { float v; asm volatile("v_accvgpr_read_b32 %0, a107" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<108>() { float v; asm volatile("v_accvgpr_read_b32 %0, a108" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<109>() { float v; asm volatile("v_accvgpr_read_b32 %0, a109" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<110>() { float v; asm volatile("v_accvgpr_read_b32 %0, a110" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<111>() { float v; asm volatile("v_accvgpr_read_b32 %0, a111" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<112>() { float v; asm volatile("v_accvgpr_read_b32 %0, a112" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<113>() { float v; asm volatile("v_accvgpr_read_b32 %0, a113" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<114>() { float v; asm volatile("v_accvgpr_read_b32 %0, a114" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<115>() { float v; asm volatile("v_accvgpr_read_b32 %0, a115" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<116>() { float v; asm volatile("v_accvgpr_read_b32 %0, a116" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<117>() { float v; asm volatile("v_accvgpr_read_b32 %0, a117" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<118>() { float v; asm volatile("v_accvgpr_read_b32 %0, a118" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<119>() { float v; asm volatile("v_accvgpr_read_b32 %0, a119" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<120>() { float v; asm volatile("v_accvgpr_read_b32 %0, a120" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<121>() { float v; asm volatile("v_accvgpr_read_b32 %0, a121" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<122>() { float v; asm volatile("v_accvgpr_read_b32 %0, a122" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<123>() { float v; asm volatile("v_accvgpr_read_b32 %0, a123" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<124>() { float v; asm volatile("v_accvgpr_read_b32 %0, a124" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<125>() { float v; asm volatile("v_accvgpr_read_b32 %0, a125" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<126>() { float v; asm volatile("v_accvgpr_read_b32 %0, a126" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<127>() { float v; asm volatile("v_accvgpr_read_b32 %0, a127" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<128>() { float v; asm volatile("v_accvgpr_read_b32 %0, a128" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<129>() { float v; asm volatile("v_accvgpr_read_b32 %0, a129" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<130>() { float v; asm volatile("v_accvgpr_read_b32 %0, a130" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<131>() { float v; asm volatile("v_accvgpr_read_b32 %0, a131" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<132>() { float v; asm volatile("v_accvgpr_read_b32 %0, a132" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<133>() { float v; asm volatile("v_accvgpr_read_b32 %0, a133" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<134>() { float v; asm volatile("v_accvgpr_read_b32 %0, a134" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<135>() { float v; asm volatile("v_accvgpr_read_b32 %0, a135" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<136>() { float v; asm volatile("v_accvgpr_read_b32 %0, a136" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<137>() { float v; asm volatile("v_accvgpr_read_b32 %0, a137" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<138>() { float v; asm volatile("v_accvgpr_read_b32 %0, a138" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<139>() { float v; asm volatile("v_accvgpr_read_b32 %0, a139" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<140>() { float v; asm volatile("v_accvgpr_read_b32 %0, a140" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<141>() { float v; asm volatile("v_accvgpr_read_b32 %0, a141" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<142>() { float v; asm volatile("v_accvgpr_read_b32 %0, a142" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<143>() { float v; asm volatile("v_accvgpr_read_b32 %0, a143" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<144>() { float v; asm volatile("v_accvgpr_read_b32 %0, a144" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<145>() { float v; asm volatile("v_accvgpr_read_b32 %0, a145" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<146>() { float v; asm volatile("v_accvgpr_read_b32 %0, a146" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<147>() { float v; asm volatile("v_accvgpr_read_b32 %0, a147" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<148>() { float v; asm volatile("v_accvgpr_read_b32 %0, a148" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<149>() { float v; asm volatile("v_accvgpr_read_b32 %0, a149" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<150>() { float v; asm volatile("v_accvgpr_read_b32 %0, a150" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<151>() { float v; asm volatile("v_accvgpr_read_b32 %0, a151" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<152>() { float v; asm volatile("v_accvgpr_read_b32 %0, a152" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<153>() { float v; asm volatile("v_accvgpr_read_b32 %0, a153" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<154>() { float v; asm volatile("v_accvgpr_read_b32 %0, a154" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<155>() { float v; asm volatile("v_accvgpr_read_b32 %0, a155" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<156>() { float v; asm volatile("v_accvgpr_read_b32 %0, a156" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<157>() { float v; asm volatile("v_accvgpr_read_b32 %0, a157" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<158>() { float v; asm volatile("v_accvgpr_read_b32 %0, a158" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<159>() { float v; asm volatile("v_accvgpr_read_b32 %0, a159" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<160>() { float v; asm volatile("v_accvgpr_read_b32 %0, a160" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<161>() { float v; asm volatile("v_accvgpr_read_b32 %0, a161" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<162>() { float v; asm volatile("v_accvgpr_read_b32 %0, a162" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<163>() { float v; asm volatile("v_accvgpr_read_b32 %0, a163" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<164>() { float v; asm volatile("v_accvgpr_read_b32 %0, a164" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<165>() { float v; asm volatile("v_accvgpr_read_b32 %0, a165" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<166>() { float v; asm volatile("v_accvgpr_read_b32 %0, a166" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<167>() { float v; asm volatile("v_accvgpr_read_b32 %0, a167" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<168>() { float v; asm volatile("v_accvgpr_read_b32 %0, a168" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<169>() { float v; asm volatile("v_accvgpr_read_b32 %0, a169" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<170>() { float v; asm volatile("v_accvgpr_read_b32 %0, a170" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<171>() { float v; asm volatile("v_accvgpr_read_b32 %0, a171" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<172>() { float v; asm volatile("v_accvgpr_read_b32 %0, a172" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<173>() { float v; asm volatile("v_accvgpr_read_b32 %0, a173" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<174>() { float v; asm volatile("v_accvgpr_read_b32 %0, a174" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<175>() { float v; asm volatile("v_accvgpr_read_b32 %0, a175" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<176>() { float v; asm volatile("v_accvgpr_read_b32 %0, a176" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<177>() { float v; asm volatile("v_accvgpr_read_b32 %0, a177" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<178>() { float v; asm volatile("v_accvgpr_read_b32 %0, a178" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<179>() { float v; asm volatile("v_accvgpr_read_b32 %0, a179" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<180>() { float v; asm volatile("v_accvgpr_read_b32 %0, a180" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<181>() { float v; asm volatile("v_accvgpr_read_b32 %0, a181" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<182>() { float v; asm volatile("v_accvgpr_read_b32 %0, a182" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<183>() { float v; asm volatile("v_accvgpr_read_b32 %0, a183" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<184>() { float v; asm volatile("v_accvgpr_read_b32 %0, a184" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<185>() { float v; asm volatile("v_accvgpr_read_b32 %0, a185" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<186>() { float v; asm volatile("v_accvgpr_read_b32 %0, a186" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<187>() { float v; asm volatile("v_accvgpr_read_b32 %0, a187" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<188>() { float v; asm volatile("v_accvgpr_read_b32 %0, a188" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<189>() { float v; asm volatile("v_accvgpr_read_b32 %0, a189" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<190>() { float v; asm volatile("v_accvgpr_read_b32 %0, a190" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<191>() { float v; asm volatile("v_accvgpr_read_b32 %0, a191" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<192>() { float v; asm volatile("v_accvgpr_read_b32 %0, a192" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<193>() { float v; asm volatile("v_accvgpr_read_b32 %0, a193" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<194>() { float v; asm volatile("v_accvgpr_read_b32 %0, a194" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<195>() { float v; asm volatile("v_accvgpr_read_b32 %0, a195" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<196>() { float v; asm volatile("v_accvgpr_read_b32 %0, a196" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<197>() { float v; asm volatile("v_accvgpr_read_b32 %0, a197" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<198>() { float v; asm volatile("v_accvgpr_read_b32 %0, a198" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<199>() { float v; asm volatile("v_accvgpr_read_b32 %0, a199" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<200>() { float v; asm volatile("v_accvgpr_read_b32 %0, a200" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<201>() { float v; asm volatile("v_accvgpr_read_b32 %0, a201" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<202>() { float v; asm volatile("v_accvgpr_read_b32 %0, a202" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<203>() { float v; asm volatile("v_accvgpr_read_b32 %0, a203" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<204>() { float v; asm volatile("v_accvgpr_read_b32 %0, a204" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<205>() { float v; asm volatile("v_accvgpr_read_b32 %0, a205" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<206>() { float v; asm volatile("v_accvgpr_read_b32 %0, a206" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<207>() { float v; asm volatile("v_accvgpr_read_b32 %0, a207" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<208>() { float v; asm volatile("v_accvgpr_read_b32 %0, a208" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<209>() { float v; asm volatile("v_accvgpr_read_b32 %0, a209" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<210>() { float v; asm volatile("v_accvgpr_read_b32 %0, a210" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<211>() { float v; asm volatile("v_accvgpr_read_b32 %0, a211" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<212>() { float v; asm volatile("v_accvgpr_read_b32 %0, a212" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<213>() { float v; asm volatile("v_accvgpr_read_b32 %0, a213" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<214>() { float v; asm volatile("v_accvgpr_read_b32 %0, a214" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<215>() { float v; asm volatile("v_accvgpr_read_b32 %0, a215" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<216>() { float v; asm volatile("v_accvgpr_read_b32 %0, a216" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<217>() { float v; asm volatile("v_accvgpr_read_b32 %0, a217" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<218>() { float v; asm volatile("v_accvgpr_read_b32 %0, a218" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<219>() { float v; asm volatile("v_accvgpr_read_b32 %0, a219" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<220>() { float v; asm volatile("v_accvgpr_read_b32 %0, a220" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<221>() { float v; asm volatile("v_accvgpr_read_b32 %0, a221" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<222>() { float v; asm volatile("v_accvgpr_read_b32 %0, a222" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<223>() { float v; asm volatile("v_accvgpr_read_b32 %0, a223" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<224>() { float v; asm volatile("v_accvgpr_read_b32 %0, a224" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<225>() { float v; asm volatile("v_accvgpr_read_b32 %0, a225" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<226>() { float v; asm volatile("v_accvgpr_read_b32 %0, a226" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<227>() { float v; asm volatile("v_accvgpr_read_b32 %0, a227" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<228>() { float v; asm volatile("v_accvgpr_read_b32 %0, a228" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<229>() { float v; asm volatile("v_accvgpr_read_b32 %0, a229" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<230>() { float v; asm volatile("v_accvgpr_read_b32 %0, a230" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<231>() { float v; asm volatile("v_accvgpr_read_b32 %0, a231" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<232>() { float v; asm volatile("v_accvgpr_read_b32 %0, a232" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<233>() { float v; asm volatile("v_accvgpr_read_b32 %0, a233" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<234>() { float v; asm volatile("v_accvgpr_read_b32 %0, a234" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<235>() { float v; asm volatile("v_accvgpr_read_b32 %0, a235" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<236>() { float v; asm volatile("v_accvgpr_read_b32 %0, a236" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<237>() { float v; asm volatile("v_accvgpr_read_b32 %0, a237" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<238>() { float v; asm volatile("v_accvgpr_read_b32 %0, a238" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<239>() { float v; asm volatile("v_accvgpr_read_b32 %0, a239" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<240>() { float v; asm volatile("v_accvgpr_read_b32 %0, a240" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<241>() { float v; asm volatile("v_accvgpr_read_b32 %0, a241" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<242>() { float v; asm volatile("v_accvgpr_read_b32 %0, a242" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<243>() { float v; asm volatile("v_accvgpr_read_b32 %0, a243" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<244>() { float v; asm volatile("v_accvgpr_read_b32 %0, a244" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<245>() { float v; asm volatile("v_accvgpr_read_b32 %0, a245" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<246>() { float v; asm volatile("v_accvgpr_read_b32 %0, a246" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<247>() { float v; asm volatile("v_accvgpr_read_b32 %0, a247" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<248>() { float v; asm volatile("v_accvgpr_read_b32 %0, a248" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<249>() { float v; asm volatile("v_accvgpr_read_b32 %0, a249" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<250>() { float v; asm volatile("v_accvgpr_read_b32 %0, a250" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<251>() { float v; asm volatile("v_accvgpr_read_b32 %0, a251" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<252>() { float v; asm volatile("v_accvgpr_read_b32 %0, a252" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<253>() { float v; asm volatile("v_accvgpr_read_b32 %0, a253" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<254>() { float v; asm volatile("v_accvgpr_read_b32 %0, a254" : "=v"(v)); return v; }
template <> __device__ __forceinline__ float agpr_read<255>() { float v; asm volatile("v_accvgpr_read_b32 %0, a255" : "=v"(v)); return v; }

// writes zero to all 256 AGPRs (and makes the register allocation of the kernel include them)
__device__ __forceinline__ void agpr_clear_all() {
  asm volatile("v_accvgpr_write_b32 a0, 0\n\tv_accvgpr_write_b32 a1, 0\n\tv_accvgpr_write_b32 a2, 0\n\tv_accvgpr_write_b32 a3, 0\n\tv_accvgpr_write_b32 a4, 0\n\tv_accvgpr_write_b32 a5, 0\n\tv_accvgpr_write_b32 a6, 0\n\tv_accvgpr_write_b32 a7, 0\n\tv_accvgpr_write_b32 a8, 0\n\tv_accvgpr_write_b32 a9, 0\n\tv_accvgpr_write_b32 a10, 0\n\tv_accvgpr_write_b32 a11, 0\n\tv_accvgpr_write_b32 a12, 0\n\tv_accvgpr_write_b32 a13, 0\n\tv_accvgpr_write_b32 a14, 0\n\tv_accvgpr_write_b32 a15, 0\n\tv_accvgpr_write_b32 a16, 0\n\tv_accvgpr_write_b32 a17, 0\n\tv_accvgpr_write_b32 a18, 0\n\tv_accvgpr_write_b32 a19, 0\n\tv_accvgpr_write_b32 a20, 0\n\tv_accvgpr_write_b32 a21, 0\n\tv_accvgpr_write_b32 a22, 0\n\tv_accvgpr_write_b32 a23, 0\n\tv_accvgpr_write_b32 a24, 0\n\tv_accvgpr_write_b32 a25, 0\n\tv_accvgpr_write_b32 a26, 0\n\tv_accvgpr_write_b32 a27, 0\n\tv_accvgpr_write_b32 a28, 0\n\tv_accvgpr_write_b32 a29, 0\n\tv_accvgpr_write_b32 a30, 0\n\tv_accvgpr_write_b32 a31, 0" ::: "a0", "a1", "a2", "a3", "a4", "a5", "a6", "a7", "a8", "a9", "a10", "a11", "a12", "a13", "a14", "a15", "a16", "a17", "a18", "a19", "a20", "a21", "a22", "a23", "a24", "a25", "a26", "a27", "a28", "a29", "a30", "a31");
  asm volatile("v_accvgpr_write_b32 a32, 0\n\tv_accvgpr_write_b32 a33, 0\n\tv_accvgpr_write_b32 a34, 0\n\tv_accvgpr_write_b32 a35, 0\n\tv_accvgpr_write_b32 a36, 0\n\tv_accvgpr_write_b32 a37, 0\n\tv_accvgpr_write_b32 a38, 0\n\tv_accvgpr_write_b32 a39, 0\n\tv_accvgpr_write_b32 a40, 0\n\tv_accvgpr_write_b32 a41, 0\n\tv_accvgpr_write_b32 a42, 0\n\tv_accvgpr_write_b32 a43, 0\n\tv_accvgpr_write_b32 a44, 0\n\tv_accvgpr_write_b32 a45, 0\n\tv_accvgpr_write_b32 a46, 0\n\tv_accvgpr_write_b32 a47, 0\n\tv_accvgpr_write_b32 a48, 0\n\tv_accvgpr_write_b32 a49, 0\n\tv_accvgpr_write_b32 a50, 0\n\tv_accvgpr_write_b32 a51, 0\n\tv_accvgpr_write_b32 a52, 0\n\tv_accvgpr_write_b32 a53, 0\n\tv_accvgpr_write_b32 a54, 0\n\tv_accvgpr_write_b32 a55, 0\n\tv_accvgpr_write_b32 a56, 0\n\tv_accvgpr_write_b32 a57, 0\n\tv_accvgpr_write_b32 a58, 0\n\tv_accvgpr_write_b32 a59, 0\n\tv_accvgpr_write_b32 a60, 0\n\tv_accvgpr_write_b32 a61, 0\n\tv_accvgpr_write_b32 a62, 0\n\tv_accvgpr_write_b32 a63, 0" ::: "a32", "a33", "a34", "a35", "a36", "a37", "a38", "a39", "a40", "a41", "a42", "a43", "a44", "a45", "a46", "a47", "a48", "a49", "a50", "a51", "a52", "a53", "a54", "a55", "a56", "a57", "a58", "a59", "a60", "a61", "a62", "a63");
  asm volatile("v_accvgpr_write_b32 a64, 0\n\tv_accvgpr_write_b32 a65, 0\n\tv_accvgpr_write_b32 a66, 0\n\tv_accvgpr_write_b32 a67, 0\n\tv_accvgpr_write_b32 a68, 0\n\tv_accvgpr_write_b32 a69, 0\n\tv_accvgpr_write_b32 a70, 0\n\tv_accvgpr_write_b32 a71, 0\n\tv_accvgpr_write_b32 a72, 0\n\tv_accvgpr_write_b32 a73, 0\n\tv_accvgpr_write_b32 a74, 0\n\tv_accvgpr_write_b32 a75, 0\n\tv_accvgpr_write_b32 a76, 0\n\tv_accvgpr_write_b32 a77, 0\n\tv_accvgpr_write_b32 a78, 0\n\tv_accvgpr_write_b32 a79, 0\n\tv_accvgpr_write_b32 a80, 0\n\tv_accvgpr_write_b32 a81, 0\n\tv_accvgpr_write_b32 a82, 0\n\tv_accvgpr_write_b32 a83, 0\n\tv_accvgpr_write_b32 a84, 0\n\tv_accvgpr_write_b32 a85, 0\n\tv_accvgpr_write_b32 a86, 0\n\tv_accvgpr_write_b32 a87, 0\n\tv_accvgpr_write_b32 a88, 0\n\tv_accvgpr_write_b32 a89, 0\n\tv_accvgpr_write_b32 a90, 0\n\tv_accvgpr_write_b32 a91, 0\n\tv_accvgpr_write_b32 a92, 0\n\tv_accvgpr_write_b32 a93, 0\n\tv_accvgpr_write_b32 a94, 0\n\tv_accvgpr_write_b32 a95, 0" ::: "a64", "a65", "a66", "a67", "a68", "a69", "a70", "a71", "a72", "a73", "a74", "a75", "a76", "a77", "a78", "a79", "a80", "a81", "a82", "a83", "a84", "a85", "a86", "a87", "a88", "a89", "a90", "a91", "a92", "a93", "a94", "a95");
  asm volatile("v_accvgpr_write_b32 a96, 0\n\tv_accvgpr_write_b32 a97, 0\n\tv_accvgpr_write_b32 a98, 0\n\tv_accvgpr_write_b32 a99, 0\n\tv_accvgpr_write_b32 a100, 0\n\tv_accvgpr_write_b32 a101, 0\n\tv_accvgpr_write_b32 a102, 0\n\tv_accvgpr_write_b32 a103, 0\n\tv_accvgpr_write_b32 a104, 0\n\tv_accvgpr_write_b32 a105, 0\n\tv_accvgpr_write_b32 a106, 0\n\tv_accvgpr_write_b32 a107, 0\n\tv_accvgpr_write_b32 a108, 0\n\tv_accvgpr_write_b32 a109, 0\n\tv_accvgpr_write_b32 a110, 0\n\tv_accvgpr_write_b32 a111, 0\n\tv_accvgpr_write_b32 a112, 0\n\tv_accvgpr_write_b32 a113, 0\n\tv_accvgpr_write_b32 a114, 0\n\tv_accvgpr_write_b32 a115, 0\n\tv_accvgpr_write_b32 a116, 0\n\tv_accvgpr_write_b32 a117, 0\n\tv_accvgpr_write_b32 a118, 0\n\tv_accvgpr_write_b32 a119, 0\n\tv_accvgpr_write_b32 a120, 0\n\tv_accvgpr_write_b32 a121, 0\n\tv_accvgpr_write_b32 a122, 0\n\tv_accvgpr_write_b32 a123, 0\n\tv_accvgpr_write_b32 a124, 0\n\tv_accvgpr_write_b32 a125, 0\n\tv_accvgpr_write_b32 a126, 0\n\tv_accvgpr_write_b32 a127, 0" ::: "a96", "a97", "a98", "a99", "a100", "a101", "a102", "a103", "a104", "a105", "a106", "a107", "a108", "a109", "a110", "a111", "a112", "a113", "a114", "a115", "a116", "a117", "a118", "a119", "a120", "a121", "a122", "a123", "a124", "a125", "a126", "a127");
  asm volatile("v_accvgpr_write_b32 a128, 0\n\tv_accvgpr_write_b32 a129, 0\n\tv_accvgpr_write_b32 a130, 0\n\tv_accvgpr_write_b32 a131, 0\n\tv_accvgpr_write_b32 a132, 0\n\tv_accvgpr_write_b32 a133, 0\n\tv_accvgpr_write_b32 a134, 0\n\tv_accvgpr_write_b32 a135, 0\n\tv_accvgpr_write_b32 a136, 0\n\tv_accvgpr_write_b32 a137, 0\n\tv_accvgpr_write_b32 a138, 0\n\tv_accvgpr_write_b32 a139, 0\n\tv_accvgpr_write_b32 a140, 0\n\tv_accvgpr_write_b32 a141, 0\n\tv_accvgpr_write_b32 a142, 0\n\tv_accvgpr_write_b32 a143, 0\n\tv_accvgpr_write_b32 a144, 0\n\tv_accvgpr_write_b32 a145, 0\n\tv_accvgpr_write_b32 a146, 0\n\tv_accvgpr_write_b32 a147, 0\n\tv_accvgpr_write_b32 a148, 0\n\tv_accvgpr_write_b32 a149, 0\n\tv_accvgpr_write_b32 a150, 0\n\tv_accvgpr_write_b32 a151, 0\n\tv_accvgpr_write_b32 a152, 0\n\tv_accvgpr_write_b32 a153, 0\n\tv_accvgpr_write_b32 a154, 0\n\tv_accvgpr_write_b32 a155, 0\n\tv_accvgpr_write_b32 a156, 0\n\tv_accvgpr_write_b32 a157, 0\n\tv_accvgpr_write_b32 a158, 0\n\tv_accvgpr_write_b32 a159, 0" ::: "a128", "a129", "a130", "a131", "a132", "a133", "a134", "a135", "a136", "a137", "a138", "a139", "a140", "a141", "a142", "a143", "a144", "a145", "a146", "a147", "a148", "a149", "a150", "a151", "a152", "a153", "a154", "a155", "a156", "a157", "a158", "a159");
  asm volatile("v_accvgpr_write_b32 a160, 0\n\tv_accvgpr_write_b32 a161, 0\n\tv_accvgpr_write_b32 a162, 0\n\tv_accvgpr_write_b32 a163, 0\n\tv_accvgpr_write_b32 a164, 0\n\tv_accvgpr_write_b32 a165, 0\n\tv_accvgpr_write_b32 a166, 0\n\tv_accvgpr_write_b32 a167, 0\n\tv_accvgpr_write_b32 a168, 0\n\tv_accvgpr_write_b32 a169, 0\n\tv_accvgpr_write_b32 a170, 0\n\tv_accvgpr_write_b32 a171, 0\n\tv_accvgpr_write_b32 a172, 0\n\tv_accvgpr_write_b32 a173, 0\n\tv_accvgpr_write_b32 a174, 0\n\tv_accvgpr_write_b32 a175, 0\n\tv_accvgpr_write_b32 a176, 0\n\tv_accvgpr_write_b32 a177, 0\n\tv_accvgpr_write_b32 a178, 0\n\tv_accvgpr_write_b32 a179, 0\n\tv_accvgpr_write_b32 a180, 0\n\tv_accvgpr_write_b32 a181, 0\n\tv_accvgpr_write_b32 a182, 0\n\tv_accvgpr_write_b32 a183, 0\n\tv_accvgpr_write_b32 a184, 0\n\tv_accvgpr_write_b32 a185, 0\n\tv_accvgpr_write_b32 a186, 0\n\tv_accvgpr_write_b32 a187, 0\n\tv_accvgpr_write_b32 a188, 0\n\tv_accvgpr_write_b32 a189, 0\n\tv_accvgpr_write_b32 a190, 0\n\tv_accvgpr_write_b32 a191, 0" ::: "a160", "a161", "a162", "a163", "a164", "a165", "a166", "a167", "a168", "a169", "a170", "a171", "a172", "a173", "a174", "a175", "a176", "a177", "a178", "a179", "a180", "a181", "a182", "a183", "a184", "a185", "a186", "a187", "a188", "a189", "a190", "a191");
  asm volatile("v_accvgpr_write_b32 a192, 0\n\tv_accvgpr_write_b32 a193, 0\n\tv_accvgpr_write_b32 a194, 0\n\tv_accvgpr_write_b32 a195, 0\n\tv_accvgpr_write_b32 a196, 0\n\tv_accvgpr_write_b32 a197, 0\n\tv_accvgpr_write_b32 a198, 0\n\tv_accvgpr_write_b32 a199, 0\n\tv_accvgpr_write_b32 a200, 0\n\tv_accvgpr_write_b32 a201, 0\n\tv_accvgpr_write_b32 a202, 0\n\tv_accvgpr_write_b32 a203, 0\n\tv_accvgpr_write_b32 a204, 0\n\tv_accvgpr_write_b32 a205, 0\n\tv_accvgpr_write_b32 a206, 0\n\tv_accvgpr_write_b32 a207, 0\n\tv_accvgpr_write_b32 a208, 0\n\tv_accvgpr_write_b32 a209, 0\n\tv_accvgpr_write_b32 a210, 0\n\tv_accvgpr_write_b32 a211, 0\n\tv_accvgpr_write_b32 a212, 0\n\tv_accvgpr_write_b32 a213, 0\n\tv_accvgpr_write_b32 a214, 0\n\tv_accvgpr_write_b32 a215, 0\n\tv_accvgpr_write_b32 a216, 0\n\tv_accvgpr_write_b32 a217, 0\n\tv_accvgpr_write_b32 a218, 0\n\tv_accvgpr_write_b32 a219, 0\n\tv_accvgpr_write_b32 a220, 0\n\tv_accvgpr_write_b32 a221, 0\n\tv_accvgpr_write_b32 a222, 0\n\tv_accvgpr_write_b32 a223, 0" ::: "a192", "a193", "a194", "a195", "a196", "a197", "a198", "a199", "a200", "a201", "a202", "a203", "a204", "a205", "a206", "a207", "a208", "a209", "a210", "a211", "a212", "a213", "a214", "a215", "a216", "a217", "a218", "a219", "a220", "a221", "a222", "a223");
  asm volatile("v_accvgpr_write_b32 a224, 0\n\tv_accvgpr_write_b32 a225, 0\n\tv_accvgpr_write_b32 a226, 0\n\tv_accvgpr_write_b32 a227, 0\n\tv_accvgpr_write_b32 a228, 0\n\tv_accvgpr_write_b32 a229, 0\n\tv_accvgpr_write_b32 a230, 0\n\tv_accvgpr_write_b32 a231, 0\n\tv_accvgpr_write_b32 a232, 0\n\tv_accvgpr_write_b32 a233, 0\n\tv_accvgpr_write_b32 a234, 0\n\tv_accvgpr_write_b32 a235, 0\n\tv_accvgpr_write_b32 a236, 0\n\tv_accvgpr_write_b32 a237, 0\n\tv_accvgpr_write_b32 a238, 0\n\tv_accvgpr_write_b32 a239, 0\n\tv_accvgpr_write_b32 a240, 0\n\tv_accvgpr_write_b32 a241, 0\n\tv_accvgpr_write_b32 a242, 0\n\tv_accvgpr_write_b32 a243, 0\n\tv_accvgpr_write_b32 a244, 0\n\tv_accvgpr_write_b32 a245, 0\n\tv_accvgpr_write_b32 a246, 0\n\tv_accvgpr_write_b32 a247, 0\n\tv_accvgpr_write_b32 a248, 0\n\tv_accvgpr_write_b32 a249, 0\n\tv_accvgpr_write_b32 a250, 0\n\tv_accvgpr_write_b32 a251, 0\n\tv_accvgpr_write_b32 a252, 0\n\tv_accvgpr_write_b32 a253, 0\n\tv_accvgpr_write_b32 a254, 0\n\tv_accvgpr_write_b32 a255, 0" ::: "a224", "a225", "a226", "a227", "a228", "a229", "a230", "a231", "a232", "a233", "a234", "a235", "a236", "a237", "a238", "a239", "a240", "a241", "a242", "a243", "a244", "a245", "a246", "a247", "a248", "a249", "a250", "a251", "a252", "a253", "a254", "a255");
}

}  // namespace gpts
