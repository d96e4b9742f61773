// Accumulation registers (AGPRs) addressed by number.
//
// The 64-rows-per-wave attention kernel keeps its O^T accumulators in fixed
// accumulation registers a0 .. a127 for the whole kernel: tuple t (16
// registers) is a[16t : 16t+15].  Only the instructions below touch them, so
// the register allocator never has to move them (it otherwise shuttles
// accumulators between the two register files inside the loop).  Every
// statement names the registers it writes as clobbers; the compiler must not
// keep anything of its own in a0 .. a127 (the kernel needs no spills, and the
// build test checks that no compiler-generated instruction names one).
//
// Hazards are the caller's: the compiler does not know that acc_pv is an MFMA,
// so after the last acc_pv and before acc_read / acc_scale the caller waits
// for the matrix pipe (mfma_drain), and after acc_zero / acc_scale it leaves
// a few cycles before the next acc_pv.
#pragma once
#include <hip/hip_runtime.h>

namespace prism {

typedef __attribute__((ext_vector_type(8))) __bf16 acc_bf16x8;

template <int N> __device__ __forceinline__ float acc_read();
template <int N> __device__ __forceinline__ void acc_write(float x);
template <int T> __device__ __forceinline__ void acc_pv(acc_bf16x8 a, acc_bf16x8 b);

#define PRISM_ACC_REG(n) \
  template <> __device__ __forceinline__ float acc_read<n>() { float x; __asm__ volatile("v_accvgpr_read_b32 %0, a" #n : "=v"(x)); return x; } \
  template <> __device__ __forceinline__ void acc_write<n>(float x) { __asm__ volatile("v_accvgpr_write_b32 a" #n ", %0" : : "v"(x) : "a" #n); }
PRISM_ACC_REG(0) PRISM_ACC_REG(1) PRISM_ACC_REG(2) PRISM_ACC_REG(3) PRISM_ACC_REG(4) PRISM_ACC_REG(5) PRISM_ACC_REG(6) PRISM_ACC_REG(7)
PRISM_ACC_REG(8) PRISM_ACC_REG(9) PRISM_ACC_REG(10) PRISM_ACC_REG(11) PRISM_ACC_REG(12) PRISM_ACC_REG(13) PRISM_ACC_REG(14) PRISM_ACC_REG(15)
PRISM_ACC_REG(16) PRISM_ACC_REG(17) PRISM_ACC_REG(18) PRISM_ACC_REG(19) PRISM_ACC_REG(20) PRISM_ACC_REG(21) PRISM_ACC_REG(22) PRISM_ACC_REG(23)
PRISM_ACC_REG(24) PRISM_ACC_REG(25) PRISM_ACC_REG(26) PRISM_ACC_REG(27) PRISM_ACC_REG(28) PRISM_ACC_REG(29) PRISM_ACC_REG(30) PRISM_ACC_REG(31)
PRISM_ACC_REG(32) PRISM_ACC_REG(33) PRISM_ACC_REG(34) PRISM_ACC_REG(35) PRISM_ACC_REG(36) PRISM_ACC_REG(37) PRISM_ACC_REG(38) PRISM_ACC_REG(39)
PRISM_ACC_REG(40) PRISM_ACC_REG(41) PRISM_ACC_REG(42) PRISM_ACC_REG(43) PRISM_ACC_REG(44) PRISM_ACC_REG(45) PRISM_ACC_REG(46) PRISM_ACC_REG(47)
PRISM_ACC_REG(48) PRISM_ACC_REG(49) PRISM_ACC_REG(50) PRISM_ACC_REG(51) PRISM_ACC_REG(52) PRISM_ACC_REG(53) PRISM_ACC_REG(54) PRISM_ACC_REG(55)
PRISM_ACC_REG(56) PRISM_ACC_REG(57) PRISM_ACC_REG(58) PRISM_ACC_REG(59) PRISM_ACC_REG(60) PRISM_ACC_REG(61) PRISM_ACC_REG(62) PRISM_ACC_REG(63)
PRISM_ACC_REG(64) PRISM_ACC_REG(65) PRISM_ACC_REG(66) PRISM_ACC_REG(67) PRISM_ACC_REG(68) PRISM_ACC_REG(69) PRISM_ACC_REG(70) PRISM_ACC_REG(71)
PRISM_ACC_REG(72) PRISM_ACC_REG(73) PRISM_ACC_REG(74) PRISM_ACC_REG(75) PRISM_ACC_REG(76) PRISM_ACC_REG(77) PRISM_ACC_REG(78) PRISM_ACC_REG(79)
PRISM_ACC_REG(80) PRISM_ACC_REG(81) PRISM_ACC_REG(82) PRISM_ACC_REG(83) PRISM_ACC_REG(84) PRISM_ACC_REG(85) PRISM_ACC_REG(86) PRISM_ACC_REG(87)
PRISM_ACC_REG(88) PRISM_ACC_REG(89) PRISM_ACC_REG(90) PRISM_ACC_REG(91) PRISM_ACC_REG(92) PRISM_ACC_REG(93) PRISM_ACC_REG(94) PRISM_ACC_REG(95)
PRISM_ACC_REG(96) PRISM_ACC_REG(97) PRISM_ACC_REG(98) PRISM_ACC_REG(99) PRISM_ACC_REG(100) PRISM_ACC_REG(101) PRISM_ACC_REG(102) PRISM_ACC_REG(103)
PRISM_ACC_REG(104) PRISM_ACC_REG(105) PRISM_ACC_REG(106) PRISM_ACC_REG(107) PRISM_ACC_REG(108) PRISM_ACC_REG(109) PRISM_ACC_REG(110) PRISM_ACC_REG(111)
PRISM_ACC_REG(112) PRISM_ACC_REG(113) PRISM_ACC_REG(114) PRISM_ACC_REG(115) PRISM_ACC_REG(116) PRISM_ACC_REG(117) PRISM_ACC_REG(118) PRISM_ACC_REG(119)
PRISM_ACC_REG(120) PRISM_ACC_REG(121) PRISM_ACC_REG(122) PRISM_ACC_REG(123) PRISM_ACC_REG(124) PRISM_ACC_REG(125) PRISM_ACC_REG(126) PRISM_ACC_REG(127)
#undef PRISM_ACC_REG

// O^T tuple T += A x B (v_mfma_f32_32x32x16_bf16 with the tuple as C and D)
#define PRISM_ACC_TUPLE(t, lo, hi, ...) \
  template <> __device__ __forceinline__ void acc_pv<t>(acc_bf16x8 a, acc_bf16x8 b) { \
    __asm__ volatile("v_mfma_f32_32x32x16_bf16 a[" #lo ":" #hi "], %0, %1, a[" #lo ":" #hi "]" : : "v"(a), "v"(b) : __VA_ARGS__); \
  }
PRISM_ACC_TUPLE(0, 0, 15, "a0", "a1", "a2", "a3", "a4", "a5", "a6", "a7", "a8", "a9", "a10", "a11", "a12", "a13", "a14", "a15")
PRISM_ACC_TUPLE(1, 16, 31, "a16", "a17", "a18", "a19", "a20", "a21", "a22", "a23", "a24", "a25", "a26", "a27", "a28", "a29", "a30", "a31")
PRISM_ACC_TUPLE(2, 32, 47, "a32", "a33", "a34", "a35", "a36", "a37", "a38", "a39", "a40", "a41", "a42", "a43", "a44", "a45", "a46", "a47")
PRISM_ACC_TUPLE(3, 48, 63, "a48", "a49", "a50", "a51", "a52", "a53", "a54", "a55", "a56", "a57", "a58", "a59", "a60", "a61", "a62", "a63")
PRISM_ACC_TUPLE(4, 64, 79, "a64", "a65", "a66", "a67", "a68", "a69", "a70", "a71", "a72", "a73", "a74", "a75", "a76", "a77", "a78", "a79")
PRISM_ACC_TUPLE(5, 80, 95, "a80", "a81", "a82", "a83", "a84", "a85", "a86", "a87", "a88", "a89", "a90", "a91", "a92", "a93", "a94", "a95")
PRISM_ACC_TUPLE(6, 96, 111, "a96", "a97", "a98", "a99", "a100", "a101", "a102", "a103", "a104", "a105", "a106", "a107", "a108", "a109", "a110", "a111")
PRISM_ACC_TUPLE(7, 112, 127, "a112", "a113", "a114", "a115", "a116", "a117", "a118", "a119", "a120", "a121", "a122", "a123", "a124", "a125", "a126", "a127")
#undef PRISM_ACC_TUPLE

// element r (0 .. 15) of tuple T
template <int T, int R> __device__ __forceinline__ float acc_get() { return acc_read<16 * T + R>(); }
template <int T, int R> __device__ __forceinline__ void acc_set(float x) { acc_write<16 * T + R>(x); }

}  // namespace prism
