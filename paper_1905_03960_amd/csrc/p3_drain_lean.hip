// The lean build of the drain kernel: the same source as p3_drain.hip with workgroups of four wavefronts
// (256 lanes) that are held to 128 registers a lane -- one wavefront and a quarter of the register file per
// SIMD, 60 KB of LDS -- so that a compute unit on which a drain workgroup is resident can still take
// workgroups of other kernels (Sec. 4: synchronisation overlapped with the backward pass, here with a
// backward pass that runs on the same GPU).  With so few lanes a lane keeps four loads in flight instead
// of two (measured: alone 1.54 instead of 1.94 ms on the VGG-19 set; the wide build needs 1.03).
#define P3_BLOCK 256
#define P3_RUN_CACHE 256
#define P3_LDS_BM_WORDS 1024
#define P3_NS p3_lean
#define P3_LAUNCH_SYM p3_launch_drain_lean
#define P3_OCCUPANCY_SYM p3_drain_occupancy_lean
// (four wavefronts per SIMD is how the register budget of 128 is stated; the LDS of a workgroup allows two
// workgroups a compute unit, and the compiler says so for every kernel: not a failure here)
#pragma clang diagnostic ignored "-Wpass-failed"
#define P3_KERNEL_ATTR __attribute__((amdgpu_waves_per_eu(4, 4)))
#define P3_LOADS_AHEAD 3
#include "p3_drain.hip"
