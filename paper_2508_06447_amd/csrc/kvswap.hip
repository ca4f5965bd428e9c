// Overlap-aware KV swapping (Algorithm 1, Section 4.3), taken entirely on the GPU: the candidate set comes
// from the selection kernel as a device array, the decision, the new block->slot map and the move lists are
// formed by one workgroup, and a copy kernel then moves the payloads between the GPU pool and a pinned,
// device-mapped CPU pool over the host link.  The host only enqueues two kernels; it never reads the sets.
//
// State kept by the caller (device int32 arrays):
//   slot_of_block[n_blocks]  GPU slot of an active block, -1 for a block that is not on the GPU
//   block_of_slot[n_slots]   the inverse map, -1 for a free slot
//   in_memory[n_blocks]      1 when the CPU pool holds the block's payload (B_Memory), else 0
#include "slim_common.h"

namespace slim {

constexpr int kPlanThreads = 1024;

enum { INFO_CAND = 0, INFO_OVERLAP, INFO_SWAPPED, INFO_OFFLOAD, INFO_LOAD, INFO_ERROR, INFO_FREED, INFO_WORDS = 8 };

// Exclusive prefix sum of one int per thread over the workgroup (kPlanThreads threads); total in `total`.
__device__ int plan_exclusive_scan(int v, int* wsum /*[16]*/, int& total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int inc = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        int t = __shfl_up(inc, o, 64);
        if (lane >= o) inc += t;
    }
    __syncthreads();                                     // wsum free from the previous use
    if (lane == 63) wsum[wave] = inc;
    __syncthreads();
    int base = 0, tot = 0;
    for (int i = 0; i < kPlanThreads / 64; ++i) {
        int s = wsum[i];
        if (i < wave) base += s;
        tot += s;
    }
    total = tot;
    return base + inc - v;
}

// Workspace (ints): flag[n_blocks] | in_list[n_slots] | slot_out[n_slots] | slot_in[n_slots] | move_slot[n_slots] | n_moves.
// slot_out[s] = block whose payload the copy kernel writes from slot s to the CPU pool (-1: none),
// slot_in[s]  = block whose payload it then reads from the CPU pool into slot s (-1: none),
// move_slot[0..n_moves) = the slots that have either, ascending.
__global__ void __launch_bounds__(kPlanThreads) kv_swap_plan_kernel(const int* __restrict__ candidate, int n_cand,
                                                                     int n_blocks, double gamma,
                                                                     int* __restrict__ slot_of_block,
                                                                     int* __restrict__ block_of_slot,
                                                                     int* __restrict__ in_memory, int n_slots,
                                                                     int* __restrict__ ws, int* __restrict__ info) {
    __shared__ int wsum[kPlanThreads / 64];
    __shared__ int s_cand, s_ov, s_err, s_missing;
    int* flag = ws;
    int* in_list = ws + n_blocks;
    int* slot_out = in_list + n_slots;
    int* slot_in = slot_out + n_slots;
    int* move_slot = slot_in + n_slots;
    const int tid = threadIdx.x;
    if (tid == 0) { s_cand = 0; s_ov = 0; s_err = 0; s_missing = 0; }
    __syncthreads();
    for (int b = tid; b < n_blocks; b += kPlanThreads) flag[b] = 0;
    for (int s = tid; s < n_slots; s += kPlanThreads) { slot_out[s] = -1; slot_in[s] = -1; }
    // The maps must be each other's inverse; otherwise nothing is touched (and no index below can leave its array).
    for (int s = tid; s < n_slots; s += kPlanThreads) {
        const int b = block_of_slot[s];
        if (b >= n_blocks || (b >= 0 && slot_of_block[b] != s)) atomicOr(&s_err, 8);
    }
    for (int b = tid; b < n_blocks; b += kPlanThreads) {
        const int s = slot_of_block[b];
        if (s >= n_slots || (s >= 0 && block_of_slot[s] != b)) atomicOr(&s_err, 8);
    }
    __syncthreads();
    // The candidate set: a repeated index counts once; an index outside [0, n_blocks) is an error.
    for (int i = tid; i < n_cand; i += kPlanThreads) {
        const int c = candidate[i];
        if ((unsigned)c >= (unsigned)n_blocks) { atomicOr(&s_err, 1); continue; }
        if (atomicExch(&flag[c], 1) == 0) {
            atomicAdd(&s_cand, 1);
            if (slot_of_block[c] >= 0) atomicAdd(&s_ov, 1);
            else if (!in_memory[c]) atomicAdd(&s_missing, 1);
        }
    }
    __syncthreads();
    const int nc = s_cand, nov = s_ov;
    int err = s_err;
    // overlap = |candidate ∩ active| / |candidate| in double, compared with gamma by a strict "<".
    const bool swap = err == 0 && nc > 0 && (double)nov / (double)nc < gamma;
    const int n_load = nc - nov;
    if (swap) {
        if (s_missing > 0) err |= 2;                     // a block to load is neither on the GPU nor in the CPU pool
        if (nc > n_slots) err |= 4;                      // the GPU pool cannot hold the candidate set
    }
    int n_off = 0, n_freed = 0, n_moves = 0;
    if (swap && err == 0) {
        // Blocks to load, ascending.
        int base = 0;
        for (int b0 = 0; b0 < n_blocks; b0 += kPlanThreads) {
            const int b = b0 + tid;
            const int is_in = (b < n_blocks && flag[b] && slot_of_block[b] < 0) ? 1 : 0;
            int tot;
            const int r = plan_exclusive_scan(is_in, wsum, tot) + base;
            if (is_in) in_list[r] = b;
            base += tot;
        }
        __syncthreads();
        // Slots that are free or hold a block that leaves, ascending: the i-th of them takes the i-th block to load.
        base = 0;
        for (int s0 = 0; s0 < n_slots; s0 += kPlanThreads) {
            const int s = s0 + tid;
            const int b = s < n_slots ? block_of_slot[s] : -1;
            const bool leaves = b >= 0 && !flag[b];
            const int freeable = (s < n_slots && (b < 0 || leaves)) ? 1 : 0;
            int tot;
            const int r = plan_exclusive_scan(freeable, wsum, tot) + base;
            base += tot;
            int copies = 0, arrives = 0;
            if (leaves) {
                slot_of_block[b] = -1;
                if (!in_memory[b]) { slot_out[s] = b; in_memory[b] = 1; copies = 1; }   // B_offload: not yet in the CPU pool
            }
            if (freeable) {
                const int nb_in = r < n_load ? in_list[r] : -1;
                slot_in[s] = nb_in;
                block_of_slot[s] = nb_in;
                if (nb_in >= 0) { slot_of_block[nb_in] = s; arrives = 1; }
            }
            int t1, t2, t3;
            plan_exclusive_scan(copies, wsum, t1);
            plan_exclusive_scan(leaves ? 1 : 0, wsum, t2);
            const int mv = plan_exclusive_scan(copies | arrives, wsum, t3) + n_moves;
            if (copies | arrives) move_slot[mv] = s;
            n_off += t1;
            n_freed += t2;
            n_moves += t3;
        }
    }
    if (tid == 0) {
        move_slot[n_slots] = n_moves;
        info[INFO_CAND] = nc;
        info[INFO_OVERLAP] = nov;
        info[INFO_SWAPPED] = (swap && err == 0) ? 1 : 0;
        info[INFO_OFFLOAD] = n_off;
        info[INFO_LOAD] = (swap && err == 0) ? n_load : 0;
        info[INFO_ERROR] = err;
        info[INFO_FREED] = n_freed;
        info[7] = 0;
    }
}

// A fixed, small number of workgroups walks the move list: work item = (move, chunk of the payload).  The link to
// the host, not the GPU, bounds this kernel: a read over it takes on the order of 10 us, so the rate is set by the
// bytes in flight.  32 workgroups x 256 threads x 8 x 16 bytes = 1 MiB in flight reaches about 56 GB/s on a
// PCIe 5.0 x16 link; 16 workgroups reach 42 GB/s, 64 add nothing.  One workgroup per item (thousands of waves that
// all wait on the link) would instead sit on every compute unit and stall the compute kernels that the transfer is
// meant to hide behind.
// A thread owns kSwapVecs 16-byte pieces of its chunk: it reads them from the slot (when the leaving block has to be
// offloaded) before it overwrites the same pieces with the arriving block's bytes, so a slot is read before it is
// reused without any synchronisation between threads.
constexpr int kSwapThreads = 256;
constexpr int kSwapVecs = 8;
constexpr int kSwapWorkgroups = 32;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__global__ void __launch_bounds__(kSwapThreads) kv_swap_copy_kernel(const int* __restrict__ slot_out,
                                                                    const int* __restrict__ slot_in,
                                                                    const int* __restrict__ move_slot,
                                                                    const int* __restrict__ n_moves_p,
                                                                    u32x4* __restrict__ gpu_pool,
                                                                    u32x4* __restrict__ host_pool, size_t block_vecs) {
    constexpr size_t per = (size_t)kSwapThreads * kSwapVecs;
    const size_t chunks = (block_vecs + per - 1) / per;
    const size_t n_items = (size_t)(*n_moves_p) * chunks;
    for (size_t it = blockIdx.x; it < n_items; it += gridDim.x) {
        const size_t mv = it / chunks, chunk = it - mv * chunks;
        const int s = move_slot[mv];
        const int b_out = slot_out[s], b_in = slot_in[s];
        u32x4* g = gpu_pool + (size_t)s * block_vecs;
        const size_t base = chunk * per + threadIdx.x;
        // Both directions of the link are used at once: the reads of the arriving bytes are issued before the
        // writes of the leaving ones wait for their data.
        u32x4 leaving[kSwapVecs], arriving[kSwapVecs];
        u32x4* h_out = host_pool + (size_t)(b_out >= 0 ? b_out : 0) * block_vecs;
        const u32x4* h_in = host_pool + (size_t)(b_in >= 0 ? b_in : 0) * block_vecs;
        if (b_in >= 0) {
#pragma unroll
            for (int u = 0; u < kSwapVecs; ++u) {
                const size_t o = base + (size_t)u * kSwapThreads;
                if (o < block_vecs) arriving[u] = __builtin_nontemporal_load(h_in + o);
            }
        }
        if (b_out >= 0) {
#pragma unroll
            for (int u = 0; u < kSwapVecs; ++u) {
                const size_t o = base + (size_t)u * kSwapThreads;
                if (o < block_vecs) leaving[u] = g[o];
            }
#pragma unroll
            for (int u = 0; u < kSwapVecs; ++u) {
                const size_t o = base + (size_t)u * kSwapThreads;
                if (o < block_vecs) __builtin_nontemporal_store(leaving[u], h_out + o);
            }
        }
        if (b_in >= 0) {
#pragma unroll
            for (int u = 0; u < kSwapVecs; ++u) {
                const size_t o = base + (size_t)u * kSwapThreads;
                if (o < block_vecs) g[o] = arriving[u];
            }
        }
    }
}

int launch_kv_swap(const int* candidate, int n_candidates, int n_blocks, double gamma, int* slot_of_block,
                   int* block_of_slot, int* in_memory, int n_slots, void* gpu_pool, void* host_pool,
                   size_t block_bytes, int* info, int* workspace, hipStream_t st) {
    hipLaunchKernelGGL(kv_swap_plan_kernel, dim3(1), dim3(kPlanThreads), 0, st, candidate, n_candidates, n_blocks, gamma,
                       slot_of_block, block_of_slot, in_memory, n_slots, workspace, info);
    int rc = check_launch();
    if (rc != SLIM_OK) return rc;
    const size_t block_vecs = block_bytes / 16;
    const int* slot_out = workspace + n_blocks + n_slots;
    const int* slot_in = slot_out + n_slots;
    const int* move_slot = slot_in + n_slots;
    hipLaunchKernelGGL(kv_swap_copy_kernel, dim3(kSwapWorkgroups), dim3(kSwapThreads), 0, st, slot_out, slot_in, move_slot,
                       move_slot + n_slots, (u32x4*)gpu_pool, (u32x4*)host_pool, block_vecs);
    return check_launch();
}

}  // namespace slim
