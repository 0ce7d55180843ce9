// mi_shmem, device side: the calls a HIP kernel of the caller's own makes on the registered heap.
// (HIP for gfx950 only; this header is C++ device code, the C ABI is include/mi_shmem.h.)
//
//   shmemx::Ctx      the heap as a kernel sees it; fill it on the host with shmem_device_context()
//                    (shmem_device_ctx has the same layout) and pass it to the kernel by value
//   shmemx::ptr / put / get / strided / atomic_fetch_add / atomic_compare_swap / atomic_fetch_or /
//   quiet / fence / acquire / team_barrier / barrier_all / pe_team_sync (a team of PEs: shmemx::PeTeam from
//   shmem_team_device_state(), same layout as shmem_pe_team)
//                    the one-sided operations, team-cooperative: every thread of every workgroup of the
//                    calling PE's team takes part in a put or get
//   shmemx::Gin      the interface of Listing 1 of the paper: put with SignalInc / SignalAdd / CounterInc
//                    actions, put_value, signal, flush, read / wait / reset of ID-addressed signals and
//                    counters, barrier_sync; construct it in the kernel as Gin{ctx, state, pe, wgs_per_pe}
//                    with the state from shmem_gin_device_state() (shmem_gin_state has the same layout)
//
// Launch such kernels on the stream the library was initialised with, npes * wgs_per_pe workgroups with
// PE = blockIdx.x / wgs_per_pe; a kernel that waits for a signal, a counter or a barrier needs all its
// workgroups resident at once.  examples/device_api_ring.hip is a complete program.
#pragma once
#include "mi_shmemx.hpp"      // the one-sided primitives (the library's own kernels are built on this same file)
#include "mi_shmem_gin.hpp"   // signals, counters, put with actions
