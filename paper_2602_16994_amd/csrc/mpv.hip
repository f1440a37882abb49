// mpv.hip -- kernels and C ABI of the tree-verification library (gfx950 only).
//
// Path of one mpv_verify call (all on the caller's stream):
//   init_kernel            zero counters, default the per-node results, queue the first tasks
//   node_task_kernel       persistent workgroups, about one per compute unit, that take tasks
//                          from a queue until none are left.
//                          Node task, one per (tree, internal node) the rule needs:
//                            softmax statistics of the node's target and draft rows, then,
//                            for each child in list order, the probability the child is
//                            tested with (or, Traversal, its starting weight) and the residual
//                            mass after its rejection (a V-wide reduction per child, over the
//                            row pair kept on chip).  A task starts the tasks that follow
//                            from it: SpecInfer the accepted child, Traversal the children of
//                            positive weight; tasks of trees whose outcome is settled are
//                            dropped.  With per-node debug outputs every node's task runs.
//                          Sampling task, one per tree, started by the task that settles the
//                            tree: the first wave does the uniform-dependent walk, then the
//                            workgroup draws the bonus token by inverse CDF from the residual
//                            of the stopping node.  (NSS, Naive, SpecTr: one per draw of the
//                            token-following walk.)
// mpv_block_efficiency and mpv_acceptance_rates run the same kernels with every node task and
// no uniforms (see Args::estimate); mpv_nucleus_mask is a kernel of its own (mpv_nucleus.h).
//
// Why this is the same computation as the step-by-step rules: every distribution
// either rule draws from is (p - c q)_+ / W(c) for one scalar c per node state
// (since (x_+/W - q)_+ = (x - W q)_+ / W), and each node is tested after exactly
// one possible history, so its test probability does not depend on the uniforms.

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <math.h>
#include <stdint.h>
#include <string.h>

#include <atomic>

#include "mpv.h"
#include "mpv_device.h"
#include "mpv_nucleus.h"

namespace mpv {

// ------------------------------------------------------------------ host/device tree tables

// 32-bit entries: a lookup with a wave-uniform index then compiles to a scalar load.
struct TreeDesc {
    int32_t N;
    int32_t parent[MPV_MAX_NODES];
    int32_t nchild[MPV_MAX_NODES];
    int32_t child_off[MPV_MAX_NODES];    // start of the node's children in child_list
    int32_t child_list[MPV_MAX_NODES];   // children of node 0, of node 1, ... ascending
    int32_t depth[MPV_MAX_NODES];
    int32_t postorder[MPV_MAX_NODES];    // depth-first, children (in list order) before their parent; root last
    int32_t rank[MPV_MAX_NODES];         // position of the node in postorder
    int32_t sub_lo[MPV_MAX_NODES];       // the node's subtree is postorder[sub_lo[n] .. rank[n]]
    int32_t cls[MPV_MAX_NODES];          // priority class of the node's task (see QueuePlan)
    int32_t class_off[8];                // QueuePlan::off again, for the kernels that read the tables from memory
};

constexpr int kMaxClasses = 4;
static_assert(kMaxClasses + 1 <= 8, "TreeDesc::class_off is too short");

// The task queue is one first-in-first-out queue per priority class; a free workgroup is
// given the oldest task of the lowest class that has one.  Class 0: the nodes from the root down
// to the first node that branches (every tree needs them).  Class 1: the nodes below it, which
// a settled tree no longer needs.  (More classes are possible: the dispatcher takes any number
// up to kMaxClasses.  Ranking the subtrees of the branching node by the order in which the rule
// visits them was tried and lost to plain age order: it starves the later subtrees of the
// trees that end up needing all of them, and those trees decide when the launch ends.)
struct QueuePlan {
    int32_t nclass;
    int32_t off[kMaxClasses + 1];        // class c owns queue[off[c] .. off[c+1])
    int32_t init_tail[kMaxClasses];      // entries of class c written by init_kernel
    int32_t init_slot[MPV_MAX_NODES];    // -1, or the node's index among the prequeued nodes of its class
    int32_t init_total;                  // prequeued tasks
    int32_t root_is_leaf;                // no node task at all: the sampling tasks are prequeued
    int32_t workers;                     // workgroups of the launch; the first prequeued tasks of class 0 go straight to them
    // Traversal, only what is needed, no workgroup to spare: the node where the tree branches
    // (-1: not used) first handles its first child only; the rest of its work (a second task:
    // "resumed") is started when that child's subtree, split_mask in postorder positions, turns
    // out to be rejected as a whole.
    int32_t split_node;
    unsigned long long split_mask;
};

// Per-(tree,node) scalars kept in the workspace, all double, each [B*N].
struct Workspace {
    double* At;      // log2-partition of the target row (internal nodes)
    double* Ad;      // same for the draft row
    double* cfin;    // c of the node's final state (all children rejected); SpecTr: the division factor rho* (the token is drawn from (p - rho* q)_+)
    double* aux;     // block-efficiency estimate, Naive and SpecTr: p_res at the node's token (see estimate_wave)
    double* a0;      // Traversal: weight the node starts with (kNotReady until its parent's task publishes it)
    double* atest;   // probability the node is tested with
    int32_t* queue;      // entry = tree * N + node (node task) or B * N + tree (sampling task), -1 = not written yet
    // [0] appended: tasks ever queued or started directly, [1] completed: tasks finished or cancelled,
    // [2] exit: set when nothing is left, [3] lock: held by the workgroup that is dispatching,
    // [4 + c] tail of class c: entries appended, [4 + kMaxClasses + c] head of class c: entries handed out,
    // [4 + 2 kMaxClasses] workgroups left waiting after the last round of dispatching (a hint)
    int32_t* qctl;
    int32_t* mailbox;    // [workgroups] kMailboxWaiting, or the task handed to that workgroup
    // Per tree, one bit per node at the node's position in postorder: `known` = the outcome of
    // the node's test is settled, `acc` = it is "accepted" (valid once known).  `decided` = the
    // sampling task has been queued (and, when only what the rule needs is computed, the
    // tree's remaining node tasks are cancelled).
    unsigned long long* known;
    unsigned long long* acc;
    int32_t* decided;
    int32_t* cur;        // [B] token-following walks: the node the walk has reached
    TreeDesc* tree;      // the tree tables, written by init_kernel for the kernel that follows
};

// Every field has a default (null / 0): what a call does not set stays off.
struct Args {
    const void* zt = nullptr;
    const void* zd = nullptr;
    const int32_t* tokens = nullptr;
    const float* uniforms = nullptr;
    const float* draw_uniforms = nullptr;      // walks that draw a token at every node they visit
    int32_t* accept_len = nullptr;
    int32_t* path_nodes = nullptr;
    int32_t* path_tokens = nullptr;
    int32_t* bonus = nullptr;
    uint32_t* counters = nullptr;
    float* dbg_stats = nullptr;
    float* dbg_edge = nullptr;
    float* dbg_accept = nullptr;
    float* dbg_resid = nullptr;
    int32_t B = 0, N = 0, V = 0, max_depth = 0;
    float k32 = 0.f;       // float(log2(e)/T)
    int32_t walk = 0;    // 0: the rule names the stopping node (SpecInfer, Traversal); a token is drawn at every
                     // visited node and followed if it is a child's: 1 from p (NSS), 2 after the Naive test,
                     // 3 after the SpecTr tests
    int32_t lazy = 0;    // compute only what the rule needs (off when per-node debug output is wanted: then every node task runs)
    int32_t stagger_ticks = 0;   // start-up spread of the persistent workgroups, in 10 ns ticks per step (8 steps)
    // Expected block efficiency instead of a verification (Sec. 5, Eq. 1-3): every node task runs
    // (lazy = 0), no uniforms are read, and what would be a tree's sampling task turns the per-node
    // results into reach probabilities.  reach_prob [B,N] may be null; expected [B].
    // estimate = 2: acceptance rates instead (App. C): per internal node, from its two rows and its
    // number of children alone; no tokens are read, nothing follows the node tasks.  alpha [B,N].
    int32_t estimate = 0;
    float* reach_prob = nullptr;
    float* expected = nullptr;
    float* alpha = nullptr;
};

constexpr int kTaskBlock = 512;
constexpr int kTaskUnroll = 4;
// node tasks keep a row pair on chip: per lane and row, kRegVecs 16-byte vectors in
// registers and kLdsVecs in LDS; the rest is re-read (kChunk vectors in flight)
constexpr int kRegVecs = 18;
constexpr int kLdsVecs = 9;
constexpr int kChunk = 2;
// upper bound on the polls of a dependency flag (about a second); see node_task_kernel
constexpr int kMaxSpins = 1 << 20;
// bit pattern (a NaN) of a starting weight that has not been published yet
constexpr unsigned long long kNotReady = ~0ull;
constexpr int kSampleBlock = kTaskBlock;     // sampling tasks run on the node tasks' workgroups
// wave tiles of the bonus sampler: 64 16-byte vectors; float rows have the smallest tiles
constexpr int kMaxTiles = MPV_MAX_VOCAB / (kWave * 4);
// task hand-over between the dispatcher and the workers (see "task queue")
constexpr int kMailboxWaiting = -1;                  // the workgroup is idle
constexpr int kMailboxSoon = -2;                     // the workgroup has asked ahead: it will be free shortly
constexpr int kTaskExit = -1;                         // what a worker's wait returns when all is done
constexpr int kWorkerSlots = 8;                       // mailboxes per dispatcher lane
constexpr int kMaxWorkgroups = kWave * kWorkerSlots;
constexpr int kKindAcceptance = 100;                   // node_task_kernel instantiation for the acceptance rates (see there)

// ------------------------------------------------------------------ init

// Grid: x covers the trees (and the few per-launch words), y the nodes, so that every table
// lookup by node has a workgroup-uniform index.
__global__ void init_kernel(QueuePlan q, TreeDesc tree, Workspace ws, Args a) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;      // tree, or word number
    const int n = blockIdx.y;
    {   // the tree tables for the next kernel, a few words per workgroup (the word number is the
        // same in every lane: scalar loads from the kernel arguments)
        const int* src = reinterpret_cast<const int*>(&tree);
        int* dst = reinterpret_cast<int*>(ws.tree);
        const int groups = gridDim.x * gridDim.y;
        for (int w = blockIdx.y * gridDim.x + blockIdx.x; w < static_cast<int>(sizeof(TreeDesc) / sizeof(int)); w += groups) {
            const int v = src[w];
            if (threadIdx.x == 0) dst[w] = v;
        }
    }
    if (n == 0) {
        if (i < MPV_COUNTER_COUNT) a.counters[i] = 0u;
        if (i == 0) { ws.qctl[0] = q.init_total; ws.qctl[1] = 0; ws.qctl[2] = 0; ws.qctl[3] = 0; ws.qctl[4 + 2 * kMaxClasses] = 0; }
        for (int c = 0; c < kMaxClasses; ++c)
            if (i == 0) {
                ws.qctl[4 + c] = (c < q.nclass) ? q.init_tail[c] : 0;
                ws.qctl[4 + kMaxClasses + c] = (c == 0) ? min(q.workers, q.init_tail[0]) : 0;
            }
        // every worker starts out waiting; the first class-0 entries are handed over below
        for (int w = i; w < kMaxWorkgroups; w += gridDim.x * blockDim.x)
            if (w >= q.init_tail[0]) ws.mailbox[w] = kMailboxWaiting;
        if (i < a.B) {
            // the root is never tested: it counts as accepted from the start
            ws.known[i] = 1ull << (a.N - 1);
            ws.acc[i] = 1ull << (a.N - 1);
            ws.decided[i] = 0;
            ws.cur[i] = 0;
            if (a.dbg_edge) {
                a.dbg_edge[static_cast<size_t>(i) * a.N * 2] = 1.f;
                a.dbg_edge[static_cast<size_t>(i) * a.N * 2 + 1] = 1.f;
            }
            if (q.root_is_leaf) {
                ws.queue[q.off[0] + i] = a.B * a.N + i;
                if (i < kMaxWorkgroups) ws.mailbox[i] = a.B * a.N + i;
            }
        }
    }
    if (i >= a.B) return;
    const int b = i;
    const size_t bn = static_cast<size_t>(b) * a.N + n;
    reinterpret_cast<unsigned long long*>(ws.a0)[bn] = kNotReady;
    if (a.alpha) a.alpha[bn] = 0.f;                          // leaves have no acceptance rate
    // a node no task ever reaches is tested with probability 0
    ws.atest[bn] = (n == 0) ? 1.0 : 0.0;
    ws.cfin[bn] = 0.0;
    // queue: the prequeued node tasks, node-major inside their class (the same node of
    // consecutive trees next to each other); everything else "not written yet"
    const int at = n * a.B + b;                               // this thread's share of the queue words
    if (at < q.off[q.nclass]) {
        int c = 0;
        while (c + 1 < q.nclass && at >= q.off[c + 1]) ++c;
        if (at - q.off[c] >= q.init_tail[c]) ws.queue[at] = -1;
    }
    if (q.init_slot[n] >= 0) {
        const int slot = q.init_slot[n] * a.B + b;
        ws.queue[q.off[tree.cls[n]] + slot] = b * a.N + n;
        if (tree.cls[n] == 0 && slot < kMaxWorkgroups) ws.mailbox[slot] = b * a.N + n;
    }
}

// ------------------------------------------------------------------ task queue
//
// node_task_kernel is launched with about one workgroup per compute unit; each runs tasks
// until told to exit.  A task is appended only when everything it needs has been published,
// so every queued task can run at once, on any workgroup: nothing depends on which or how
// many workgroups are resident.
//   append:   appended++, then slot = tail++ of the class, then the entry is written.
//   request:  mailbox[w] = "soon" when a workgroup asks ahead, before the last sweep of its
//             current task (the answer is then usually there when it is done), "waiting" once
//             it has nothing to do.  Idle workgroups are served before those that asked ahead.
//   dispatch: a workgroup that has nothing to do takes the dispatcher lock if it is free and,
//             with its first wave, hands queued tasks to waiting workgroups (itself included)
//             in priority order (class, then age), until it has a task of its own; then it
//             releases the lock.  Those that find the lock taken poll their mailbox.  If every
//             workgroup is busy nobody dispatches, and nobody needs to.  Node tasks of trees
//             whose outcome is settled are dropped here when only what is needed is computed.
//   end:      nothing queued and completed == appended, with appended read before and after
//             completed and unchanged: no task is queued, handed out or running, so nothing
//             can be appended any more; the dispatching workgroup sets the exit flag.  A
//             task's appends are performed before its completed++.
// A workgroup may also run a task it has produced itself straight away (counted in appended,
// never queued).  Every wait is bounded.

__device__ __forceinline__ int ld_relaxed(const int32_t* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long ld_relaxed(const unsigned long long* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_relaxed(int32_t* p, int v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// all loads, stores and atomics issued so far by this lane have been performed
__device__ __forceinline__ void wait_memory() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// One lane: ask for a task ahead of time.
__device__ __forceinline__ void request_task(const Workspace& ws) {
    st_relaxed(&ws.mailbox[blockIdx.x], kMailboxSoon);
}

// Append one task to class c (one lane).  The caller's earlier stores have been waited for.
__device__ __forceinline__ void append_task(const TreeDesc& tree, const Workspace& ws, int c, int entry) {
    (void)atomicAdd(&ws.qctl[0], 1);
    wait_memory();                                    // counted before it can be handed out (and finished)
    const int slot = atomicAdd(&ws.qctl[4 + c], 1);
    const int first = tree.class_off[c], end = tree.class_off[c + 1];
    if (slot < end - first) st_relaxed(&ws.queue[first + slot], entry);
}

// One round of dispatching, by a whole wave that holds the lock.  Lane c keeps the head of
// class c in `head`; lane l looks after the workgroups l, l + 64, ...  Returns true when
// everything is finished (the exit flag has been set).
__device__ __forceinline__ bool dispatch_round(const QueuePlan& q, const TreeDesc& tree, const Workspace& ws, const Args& a, bool drop_settled,
                               int& head, long long t_begin) {
    __shared__ int sh_head[kMaxClasses], sh_before[kMaxClasses + 1];
    const int lane = threadIdx.x;
    const int workers = static_cast<int>(gridDim.x);
    // who is waiting, what is queued
    unsigned waiting = 0u, soon = 0u;
#pragma unroll
    for (int sl = 0; sl < kWorkerSlots; ++sl) {
        const int w = lane + kWave * sl;
        if (w < workers) {
            const int m = ld_relaxed(&ws.mailbox[w]);
            if (m == kMailboxWaiting) waiting |= 1u << sl;
            if (m == kMailboxSoon) soon |= 1u << sl;
        }
    }
    const int tail = (lane < q.nclass) ? ld_relaxed(&ws.qctl[4 + lane]) : 0;
    const int avail = (lane < q.nclass) ? tail - head : 0;
    const int my_waiting = __popc(waiting), my_soon = __popc(soon);
    const int waiting_incl = wave_inclusive_scan_i32(my_waiting);
    const int soon_incl = wave_inclusive_scan_i32(my_soon);
    const int avail_incl = wave_inclusive_scan_i32(avail);
    const int total_idle = __shfl(waiting_incl, kWave - 1, kWave);
    const int total_waiting = total_idle + __shfl(soon_incl, kWave - 1, kWave);
    const int total_avail = __shfl(avail_incl, kWave - 1, kWave);
    if (total_avail == 0) {
        int done = 0;
        if (lane == 0) {
            const int a1 = ld_relaxed(&ws.qctl[0]);
            wait_memory();
            const int co = ld_relaxed(&ws.qctl[1]);
            wait_memory();
            const int a2 = ld_relaxed(&ws.qctl[0]);
            done = (co == a1 && a1 == a2) ? 1 : 0;
            // a queue entry that never arrives, a task that never ends: give up after 2 s (must never happen)
            if (!done && wall_clock64() - t_begin > 200000000ll) {
                atomicAdd(&a.counters[MPV_COUNTER_DEPENDENCY_TIMEOUT], 1u);
                done = 1;
            }
            if (done) {
                st_relaxed(&ws.qctl[2], 1);
                wait_memory();
            }
        }
        if (__builtin_amdgcn_readfirstlane(done)) return true;
    }
    // how many will still be waiting after this round: tasks look at it to decide whether work
    // that may turn out useless is worth queueing
    if (lane == 0) st_relaxed(&ws.qctl[4 + 2 * kMaxClasses], max(0, total_idle - total_avail));
    if (total_avail == 0 || total_waiting == 0) {
        __builtin_amdgcn_s_sleep(8);
        return false;
    }
    // Requester number r gets queued task number r (in class, age order); the idle workgroups
    // come first (in lane, slot order), then those that asked ahead.
    if (lane < q.nclass) { sh_head[lane] = head; sh_before[lane + 1] = avail_incl; }
    if (lane == 0) sh_before[0] = 0;
    __builtin_amdgcn_wave_barrier();
    int r_idle = waiting_incl - my_waiting;
    int r_soon = total_idle + soon_incl - my_soon;
    for (int sl = 0; sl < kWorkerSlots; ++sl) {
        int mine;
        if ((waiting >> sl) & 1u) mine = r_idle++;
        else if ((soon >> sl) & 1u) mine = r_soon++;
        else continue;
        if (mine >= total_avail) continue;
        int c = 0;
        while (mine >= sh_before[c + 1]) ++c;         // ends: mine < total_avail = sh_before[nclass]
        const int32_t* slot = &ws.queue[tree.class_off[c] + sh_head[c] + (mine - sh_before[c])];
        int entry = -1;
        for (int spin = 0; spin < kMaxSpins; ++spin) {          // the entry follows its tail count closely
            entry = ld_relaxed(slot);
            if (entry >= 0) break;
            __builtin_amdgcn_s_sleep(2);
        }
        if (entry < 0) {                              // must never happen: counted as finished, nobody runs it
            atomicAdd(&a.counters[MPV_COUNTER_DEPENDENCY_TIMEOUT], 1u);
            atomicAdd(&ws.qctl[1], 1);
        } else if (drop_settled && entry < a.B * a.N && ld_relaxed(&ws.decided[entry / a.N]) != 0) {
            atomicAdd(&a.counters[MPV_COUNTER_NODE_TASKS_CANCELLED], 1u);
            atomicAdd(&ws.qctl[1], 1);
        } else {
            st_relaxed(&ws.mailbox[lane + kWave * sl], entry);
        }
    }
    if (lane < q.nclass) {
        const int before = avail_incl - avail;
        head += max(0, min(avail, total_waiting - before));
    }
    __builtin_amdgcn_wave_barrier();                  // sh_head / sh_before are rewritten next time round
    wait_memory();
    return false;
}

// The next task of this workgroup, or kTaskExit; called by every lane of the first wave, returns
// the same value in each.  The workgroup has asked (its mailbox says "waiting" or already holds
// the answer).  `previous` is the task it took from the mailbox last: until the request has
// reached memory the mailbox may still show it (no entry is ever handed out twice, so the
// value is unambiguous).
__device__ __forceinline__ int acquire_task(const QueuePlan& q, const TreeDesc& tree, const Workspace& ws, const Args& a, int previous, bool drop_settled) {
    const int lane = threadIdx.x;
    int32_t* const box = &ws.mailbox[blockIdx.x];
    for (int spin = 0; spin < kMaxSpins; ++spin) {
        int t = 0, ex = 0, lk = 1;
        if (lane == 0) {
            // nothing to do any more: from "soon" to "waiting" (unless the answer has arrived)
            t = (spin == 0) ? static_cast<int>(atomicCAS(box, kMailboxSoon, kMailboxWaiting)) : ld_relaxed(box);
            ex = ld_relaxed(&ws.qctl[2]);
            lk = ld_relaxed(&ws.qctl[3]);
        }
        t = __builtin_amdgcn_readfirstlane(t);
        if (t >= 0 && t != previous) return t;
        if (__builtin_amdgcn_readfirstlane(ex)) return kTaskExit;
        int got = 0;
        if (lane == 0 && lk == 0) got = (atomicCAS(&ws.qctl[3], 0, 1) == 0) ? 1 : 0;
        if (__builtin_amdgcn_readfirstlane(got)) {
            // the previous holder wrote the heads before it released the lock
            int head = (lane < q.nclass) ? ld_relaxed(&ws.qctl[4 + kMaxClasses + lane]) : 0;
            const long long t_begin = wall_clock64();
            int result = kTaskExit;
            for (;;) {
                const bool finished = dispatch_round(q, tree, ws, a, drop_settled, head, t_begin);
                if (finished) break;
                int mine = (lane == 0) ? ld_relaxed(box) : 0;
                mine = __builtin_amdgcn_readfirstlane(mine);
                if (mine >= 0 && mine != previous) { result = mine; break; }
            }
            if (lane < q.nclass) st_relaxed(&ws.qctl[4 + kMaxClasses + lane], head);
            wait_memory();
            if (lane == 0) st_relaxed(&ws.qctl[3], 0);
            return result;
        }
        __builtin_amdgcn_s_sleep(8);
    }
    if (lane == 0) atomicAdd(&a.counters[MPV_COUNTER_DEPENDENCY_TIMEOUT], 1u);     // must never happen
    return kTaskExit;
}

// Results one task leaves for another task of the same launch (which may run on another
// chiplet, behind another L2 cache): written through and read past the caches with relaxed
// device-scope atomics.  Order between them is the writer's business: it waits for its stores
// to be acknowledged (s_waitcnt vmcnt(0)) before the atomic that lets the reader start.
__device__ __forceinline__ void st_shared_f64(double* p, double v) {
    __hip_atomic_store(reinterpret_cast<unsigned long long*>(p),
                       static_cast<unsigned long long>(__double_as_longlong(v)), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ double ld_shared_f64(const double* p) {
    return __longlong_as_double(static_cast<long long>(__hip_atomic_load(
        reinterpret_cast<const unsigned long long*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)));
}

// ------------------------------------------------------------------ node task

// (defined below) walk and bonus token of tree b, or one draw of a token-following walk, by the
// whole workgroup; returns the task that follows from it (-1: none; the same in every lane)
template <class E, int METHOD>
__device__ __forceinline__ int sample_task(const TreeDesc& tree, const Workspace& ws, const Args& a, int b,
                           float* tile_sum, double* scratch);

// (defined below) expected block efficiency of tree b from the per-node results, by the first wave
template <int METHOD>
__device__ __forceinline__ void estimate_wave(const TreeDesc& tree, const Workspace& ws, const Args& a, int b);

template <class E, int KIND, bool FULL>
__global__ __launch_bounds__(kTaskBlock) void node_task_kernel(QueuePlan q, Workspace ws, Args a) {
    using T = typename E::T;
    // KIND: MPV_METHOD_SPECINFER (all top-down rules) or MPV_METHOD_TRAVERSAL, or kKindAcceptance: the
    // top-down kernel reduced to what the acceptance rates need (an instantiation of its own, so that
    // its extra sweeps do not weigh on the register allocation of the verification kernels)
    constexpr bool ACCEPT = KIND == kKindAcceptance;
    constexpr int METHOD = ACCEPT ? MPV_METHOD_SPECINFER : KIND;
    __shared__ double scratch[2 * (kTaskBlock / kWave)];
    // rows too short to fill the on-chip slots are simply streamed again (they sit in L2)
    constexpr int RV = FULL ? kRegVecs : 0;
    constexpr int LV = FULL ? kLdsVecs : 0;
    constexpr int CH = FULL ? kChunk : 4;
    __shared__ uint4 lds_t[(LV > 0 ? LV : 1) * kTaskBlock];
    __shared__ uint4 lds_d[(LV > 0 ? LV : 1) * kTaskBlock];

    // the sampling task's table of tile masses shares the LDS the kept rows use
    static_assert(!FULL || sizeof(lds_t) >= kMaxTiles * sizeof(float), "tile masses do not fit in the kept-row LDS");
    __shared__ float own_tile_mass[FULL ? 1 : kMaxTiles];

    __shared__ int sh_task;
    // The tree tables are read from LDS, copied there from the workspace (init_kernel put them
    // there), not from the kernel arguments: a table that is a kernel argument and is indexed
    // with a value the compiler keeps in a vector register is copied, whole, into every lane's
    // private memory.
    __shared__ TreeDesc sh_tree;
    for (int w = threadIdx.x; w < static_cast<int>(sizeof(TreeDesc) / sizeof(int)); w += kTaskBlock)
        reinterpret_cast<int*>(&sh_tree)[w] = reinterpret_cast<const int*>(ws.tree)[w];
    const TreeDesc& tree = sh_tree;               // the task loop starts with a barrier
    // Every task alternates a memory-bound sweep with compute-bound replays and all tasks of a
    // kind take the same time, so workgroups started together stay in step: all load at once
    // (sharing the memory bandwidth), then all leave memory idle.  Spreading their start over
    // a fraction of a task keeps them out of phase for the rest of the launch.
    if (a.stagger_ticks > 0) {
        const long long wait = static_cast<long long>((blockIdx.x >> 3) & 7) * a.stagger_ticks;
        const long long t0 = wall_clock64();
        while (wall_clock64() - t0 < wait) __builtin_amdgcn_s_sleep(16);    // the clock always advances: bounded
    }
    const bool drop_settled = METHOD == MPV_METHOD_TRAVERSAL && a.lazy != 0;
    int previous_task = -3;                           // last task taken from the mailbox: none yet
    bool asked = true;                                // the launch starts with every mailbox waiting or filled
    int own_task = -1;                                // a task this workgroup produced for itself
    for (;;) {
    __syncthreads();                                  // the previous task is done with LDS
    int task;
    if (own_task >= 0) {
        task = own_task;
        own_task = -1;
    } else {
        if (threadIdx.x < kWave) {
            if (!asked) {
                if (threadIdx.x == 0) st_relaxed(&ws.mailbox[blockIdx.x], kMailboxWaiting);
                wait_memory();
            }
            const int t = acquire_task(q, tree, ws, a, previous_task, drop_settled);
            if (threadIdx.x == 0) sh_task = t;
        }
        __syncthreads();
        task = sh_task;
        previous_task = task;
        asked = false;
        if (task == kTaskExit) break;
    }
    task = __builtin_amdgcn_readfirstlane(task);
    if (task >= a.B * a.N && task < a.B * a.N + a.B) {
        // the tree's outcome is settled: walk and bonus token
        if (!asked) {
            if (threadIdx.x == 0) request_task(ws);
            asked = true;
        }
        float* tile_mass = FULL ? reinterpret_cast<float*>(lds_t) : own_tile_mass;
        int next = -1;
        if (ACCEPT) {
            // acceptance rates: nothing follows the node tasks (a root without children has none at all)
        } else if (a.estimate) {
            if (threadIdx.x < kWave) estimate_wave<METHOD>(tree, ws, a, task - a.B * a.N);
        } else {
            next = sample_task<E, METHOD>(tree, ws, a, task - a.B * a.N, tile_mass, scratch);
        }
        if (next >= 0) own_task = next;               // a token-following walk goes on
        if (threadIdx.x == 0) {
            if (next >= 0) {
                (void)atomicAdd(&ws.qctl[0], 1);
                wait_memory();                        // counted (and the walk's position written) first
            }
            atomicAdd(&ws.qctl[1], 1);
        }
        continue;
    }
    // a node task, or the resumed task of the node where the tree branches
    // (tree, node: made scalar explicitly, so that the table lookups below have uniform addresses)
    const bool resumed = task >= a.B * a.N + a.B;
    const int b = __builtin_amdgcn_readfirstlane(resumed ? task - (a.B * a.N + a.B) : task / a.N);
    const int n = __builtin_amdgcn_readfirstlane(resumed ? q.split_node : task % a.N);
    const size_t bn = static_cast<size_t>(b) * a.N + n;
    const T* zt = static_cast<const T*>(a.zt) + bn * a.V;
    const T* zd = static_cast<const T*>(a.zd) + bn * a.V;
    const int V = a.V;
    const float k32 = a.k32;

    const int k = tree.nchild[n];
    if (threadIdx.x == 0) atomicAdd(&a.counters[resumed ? MPV_COUNTER_NODE_TASKS_RESUMED : MPV_COUNTER_NODE_TASKS_RUN], 1u);
    const bool split_here = METHOD == MPV_METHOD_TRAVERSAL && a.lazy && !resumed && n == q.split_node;

    // ---- the children's tokens and this node's starting weight: fetched now, so that
    //      their latency hides behind the sweep (lane j looks after child j)
    __shared__ int ch_tok[MPV_MAX_CHILDREN];
    __shared__ float ch_zt[MPV_MAX_CHILDREN], ch_zd[MPV_MAX_CHILDREN];
    __shared__ float ch_u[MPV_MAX_CHILDREN];
    __shared__ double sh_a0;
    __shared__ float sh_un;
    int pf_x = -1;
    float pf_u = 2.f;
    if (threadIdx.x < k && a.tokens) {
        const size_t bc = static_cast<size_t>(b) * a.N + tree.child_list[tree.child_off[n] + threadIdx.x];
        pf_x = a.tokens[bc];
        if (!a.estimate) pf_u = a.uniforms[bc];
    }
    if (threadIdx.x == kWave && !a.estimate) pf_u = a.uniforms[bn];        // the node's own uniform
    // are workgroups idle (as of the last round of dispatching)?
    __shared__ int sh_idle, sh_ahead;
    int pf_idle = 0;
    if (threadIdx.x == 0) pf_idle = ld_relaxed(&ws.qctl[4 + 2 * kMaxClasses]);

    // ---- softmax statistics of both rows: the one read of the pair from memory
    RetainedPair<E, kTaskBlock, RV, LV, CH, FULL> pair;
    int tid_l = threadIdx.x;
    asm volatile("" : "+v"(tid_l));     // per-task copy: nothing derived from it is kept across tasks
    pair.setup(zt, zd, V, lds_t, lds_d, tid_l);
    pair.issue_register_loads();
    T pf_t = 0, pf_d = 0;       // kept as stored until the sweep is over: touching them now would wait for every load above
    if (pf_x >= 0 && pf_x < V) {
        pf_t = zt[pf_x];
        pf_d = zd[pf_x];
    }
    // Traversal, only what is needed, and idle workgroups about: an only child's task is queued
    // now, ahead of its starting weight.  It reads its rows while this task reads its own and
    // then finds the weight published (or waits a moment for it), so that a chain of nodes
    // takes little more than one task's time.  If the weight turns out to be 0 it gives up.
    if (threadIdx.x == 0) {
        int ahead = 0;
        if (METHOD == MPV_METHOD_TRAVERSAL && a.lazy && k == 1 && !split_here && pf_idle != 0) {
            const int cn = tree.child_list[tree.child_off[n]];
            if (tree.nchild[cn] > 0) {
                append_task(tree, ws, tree.cls[cn], b * a.N + cn);
                ahead = 1;
            }
        }
        sh_ahead = ahead;
    }
    RowStat rt, rd;
    {
        PairStatsRawF<E> f;
        f.t.init(); f.d.init(); f.k32 = k32;
        pair.first_pass(f);
        if (threadIdx.x < k) { ch_tok[threadIdx.x] = pf_x; ch_u[threadIdx.x] = pf_u; ch_zt[threadIdx.x] = E::load_one(&pf_t); ch_zd[threadIdx.x] = E::load_one(&pf_d); }
        if (threadIdx.x == kWave) sh_un = pf_u;
        if (threadIdx.x == 0) sh_idle = pf_idle;
        if (threadIdx.x == 0) {
            // Traversal: the starting weight comes from the parent's task, which published it
            // before it queued this task; the two stores may still arrive in either order.
            double a0 = 1.0;
            if (METHOD == MPV_METHOD_TRAVERSAL && n != 0) {
                // value and "ready" flag are one 64-bit word (a weight is never NaN), read and
                // written with relaxed device-scope atomics: no fence, no cache invalidation
                unsigned long long bits = kNotReady;
                for (int spin = 0; spin < kMaxSpins; ++spin) {
                    bits = __hip_atomic_load(reinterpret_cast<unsigned long long*>(&ws.a0[bn]), __ATOMIC_RELAXED,
                                             __HIP_MEMORY_SCOPE_AGENT);
                    if (bits != kNotReady) break;
                    __builtin_amdgcn_s_sleep(32);
                }
                if (bits != kNotReady) {
                    a0 = __longlong_as_double(static_cast<long long>(bits));
                } else {            // cannot happen while blocks are dispatched in index order; never hang
                    a0 = 0.0;
                    atomicAdd(&a.counters[MPV_COUNTER_DEPENDENCY_TIMEOUT], 1u);
                }
            }
            sh_a0 = a0;
        }
        finish_stats2<kTaskBlock, false>(f.t, f.d, rt, rd, scratch);     // its barriers publish the above
        rt.A = uniform_f64(rt.A);
        rd.A = uniform_f64(rd.A);
    }

    // ---- per-child scalars and one residual-mass reduction per child
    double wa = (METHOD == MPV_METHOD_TRAVERSAL) ? uniform_f64(sh_a0) : 1.0;   // node weight a
    const bool child_ahead = sh_ahead != 0;
    if (METHOD == MPV_METHOD_TRAVERSAL && a.lazy && n != 0 && !(wa > 0.0)) {
        // queued ahead of its weight, which is 0: the parent has written off the whole subtree.
        // Nothing to do but to pass the news on to an only child queued ahead in turn.
        if (threadIdx.x == 0) {
            if (child_ahead) {
                const size_t bc = static_cast<size_t>(b) * a.N + tree.child_list[tree.child_off[n]];
                __hip_atomic_store(reinterpret_cast<unsigned long long*>(&ws.a0[bc]),
                                   static_cast<unsigned long long>(__double_as_longlong(0.0)),
                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            wait_memory();
            atomicAdd(&ws.qctl[1], 1);
        }
        continue;
    }
    double c = 0.0, W = 1.0;
    const double kd = static_cast<double>(k32);
    // test outcomes this task settles, one bit per node at its position in postorder
    unsigned long long settled_bits = 0ull, accepted_bits = 0ull;
    int next_node = -1;                               // SpecInfer, only what is needed: the accepted child
    int own_child = -1;                               // Traversal: index of the first child whose task is to be run
    bool paused = false;
    bool own_given = false;                           // that child's task was queued after all (some workgroup is idle)
    const bool idle_seen = sh_idle != 0;
    // SpecTr (App. B, Alg. 3): the division factor rho* is the root of
    //   f(rho) = p_acc(rho) - rho beta(rho),  p_acc = 1 - (1 - beta)^k,  beta(rho) = sum_v min(p_v/rho, q_v)
    // on [1, k]; f decreases, f(1) >= 0 >= f(k).  Written with the sums of positive terms
    //   W(rho) = sum_v (p_v - rho q_v)_+   and   D(rho) = sum_v (q_v - p_v/rho)_+ = (W + rho - 1)/rho = 1 - beta,
    // f = W - D^k: no cancellation, so the sign of f is right even where |f| is far below the
    // rounding error of beta itself (p close to q, where f is nearly flat to the right of the root).
    // Each W is one sweep over the pair on chip, the same reduction the other rules use.  At the
    // root p_acc/beta = rho*, so the vector the token is drawn from, (p - gamma min(p/rho*, q))_+,
    // is (p - rho* q)_+ : the node's final state is simply c = rho*.
    // The paper's binary search is replaced by Newton's method from rho = 1, kept inside the
    // bracket [last rho with f > 0, first rho with f < 0] (a step that leaves it is replaced by the
    // midpoint); the sweep returns the slope with the value: W'(rho) = -sum_{p > rho q} q, and
    // D' = (W' + 1 - D)/rho.  Once a step is shorter than the tolerance the next point is put
    // just across, to close the bracket.  The same root in about seven sweeps instead of thirty
    // (f has a kink where the largest token switches sides and can be nearly flat beyond it:
    // there it takes more).
    double sp_rho = 1.0, sp_W = 1.0;
    if (METHOD == MPV_METHOD_SPECINFER && a.walk == 3) {
        constexpr double kTol = 3e-8;                 // relative width of the final bracket
        double lo = 1.0, hi = static_cast<double>(k);
        double x = 1.0, fx = 0.0, dfx = 0.0;
        const int evals = (k > 1) ? 64 : 1;
        for (int it = 0; it < evals; ++it) {
            if (it > 0) {
                double cand = 0.0;                    // outside the bracket: "no candidate"
                if (dfx < 0.0) {
                    const double step = -fx / dfx;
                    cand = x + step;
                    if (fabs(step) <= 0.5 * kTol * x) cand = fx > 0.0 ? x * (1.0 + kTol) : x * (1.0 - kTol);
                }
                if (!(cand > lo && cand < hi)) cand = 0.5 * (lo + hi);
                x = uniform_f64(cand);
            }
            const ResidualConsts rc = residual_consts(rt.A, rd.A, x);
            ResidualMassSlopeRawF<E> f;
            f.init();
            f.k32 = k32; f.nAt = rc.nAt; f.nAd = rc.nAd; f.rho = uniform_f32(rc.rho);
            pair.replay(f);
            double lane_mass = static_cast<double>(f.acc0) + static_cast<double>(f.acc1);
            double lane_draft = static_cast<double>(f.q0) + static_cast<double>(f.q1);
            block_sum2<kTaskBlock>(lane_mass, lane_draft, scratch);
            const double scale = uniform_f64(rc.scale);
            const double Wx = uniform_f64(scale * lane_mass);
            const double dWx = -uniform_f64(scale * lane_draft) / x;       // the sweep added up rho q over {p > rho q}
            const double Dx = fmin(fmax((Wx + x - 1.0) / x, 0.0), 1.0);
            const double dDx = (dWx + 1.0 - Dx) / x;
            const double kk = static_cast<double>(k);
            fx = Wx - pow(Dx, kk);
            dfx = dWx - kk * pow(Dx, kk - 1.0) * dDx;
            sp_rho = x;
            sp_W = Wx;
            if (it == 0) {
                if (!(fx > 0.0)) break;               // the root is 1 (also when k = 1)
            } else {
                if (fx > 0.0) lo = x;
                else if (fx < 0.0) hi = x;
                else break;
                if (hi - lo <= kTol * hi) break;
            }
        }
    }
    if (ACCEPT) {
        // Acceptance rate of this node (App. C): the chance that the solver's output is one of k draft
        // tokens drawn i.i.d. from q.  For SpecInfer and SpecTr the part of App. C's formulas that
        // covers a hit by the token drawn from the final residual is zero (the residual has no mass
        // where a draft token can have been rejected), which leaves 1 - (mass of that residual):
        //   SpecInfer  1 - W(c_{k+1}),  c_1 = 0, c_{i+1} = c_i + W(c_i)      (k sweeps)
        //   SpecTr     p_acc = 1 - (1 - beta(rho*))^k                          (the search above)
        //   NSS        sum_t p (1 - (1-q)^k)                                    (one sweep)
        //   Naive      sum_t min(p,q) + sum_t (p-q)_+ (1 - (1-q)^(k-1))         (one sweep)
        double alpha;
        if (a.walk == 3) {
            const double D = fmin(fmax((sp_W + sp_rho - 1.0) / sp_rho, 0.0), 1.0);
            alpha = 1.0 - pow(D, static_cast<double>(k));
        } else if (a.walk == 0) {
            double cc = 0.0, Wc = 1.0;
            for (int j = 0; j < k && Wc > 0.0; ++j) {
                cc = uniform_f64(cc + Wc);
                const ResidualConsts rc = residual_consts(rt.A, rd.A, cc);
                ResidualMassRawF<E> f;
                f.init();
                f.k32 = k32; f.nAt = rc.nAt; f.nAd = rc.nAd; f.rho = uniform_f32(rc.rho);
                pair.replay(f);
                const double lane_mass = static_cast<double>(f.acc0) + static_cast<double>(f.acc1);
                Wc = uniform_f64(uniform_f64(rc.scale) * block_sum<kTaskBlock>(lane_mass, scratch));
            }
            alpha = 1.0 - Wc;
        } else {
            AcceptanceF<E> f;
            const float At_hi = static_cast<float>(rt.A), Ad_hi = static_cast<float>(rd.A);
            f.init(k32, -At_hi, -Ad_hi, static_cast<float>(exp2(static_cast<double>(At_hi) - rt.A)),
                   static_cast<float>(exp2(static_cast<double>(Ad_hi) - rd.A)), a.walk == 1 ? k : k - 1, a.walk == 2);
            sweep_pair<E, kTaskBlock, kTaskUnroll>(zt, zd, V, f);
            const double lane_sum = static_cast<double>(f.acc0) + static_cast<double>(f.acc1);
            alpha = uniform_f64(block_sum<kTaskBlock>(lane_sum, scratch));
        }
        if (threadIdx.x == 0) {
            a.alpha[bn] = static_cast<float>(fmin(fmax(alpha, 0.0), 1.0));
            atomicAdd(&ws.qctl[1], 1);
        }
        continue;
    }
    for (int j = 0; j < k; ++j) {
        // a resumed task repeats the arithmetic of the first child (whose task has long run)
        // to get at the residual that follows its rejection
        const bool redone = resumed && j == 0;
        const int cn = tree.child_list[tree.child_off[n] + j];
        const size_t bc = static_cast<size_t>(b) * a.N + cn;
        const int x = ch_tok[j];
        double px = 0.0, qx = 0.0;
        const bool tok_ok = (x >= 0 && x < V);
        if (tok_ok) {
            px = exp2(static_cast<double>(ch_zt[j]) * kd - rt.A);
            qx = exp2(static_cast<double>(ch_zd[j]) * kd - rd.A);
        } else if (threadIdx.x == 0) {
            atomicAdd(&a.counters[MPV_COUNTER_BAD_TOKEN], 1u);
        }
        const double Px = fmax(px - c * qx, 0.0) / W;     // current distribution at x
        double w_child;
        if (METHOD == MPV_METHOD_TRAVERSAL) {
            // block-verification weight recursion (Sec. 3.1) with the current a and P
            if (!(wa > 0.0) || !(Px > 0.0)) w_child = 0.0;
            else if (qx > 0.0) w_child = fmin(1.0, wa * Px / qx);
            else w_child = 1.0;
        } else if (a.walk == 1) {
            // NSS tests nothing (App. B Alg. 1); the estimate wants p(x): the chance that Y ~ p is x
            w_child = px;
        } else if (a.walk == 3) {
            // App. B Alg. 3: accept x if rho* U <= p(x)/q(x)
            if (qx > 0.0) w_child = fmin(1.0, px / (sp_rho * qx));
            else w_child = (px > 0.0) ? 1.0 : 0.0;
        } else {
            // App. B Alg. 4: accept x with min(1, p(x)/q(x))
            if (qx > 0.0) w_child = fmin(1.0, Px / qx);
            else w_child = (Px > 0.0) ? 1.0 : 0.0;
        }
        // the same comparison the walk makes
        const bool child_accepted = static_cast<double>(ch_u[j]) < w_child;
        const unsigned long long child_bit = 1ull << tree.rank[cn];
        if (redone) {
        } else if (METHOD == MPV_METHOD_SPECINFER) {
            settled_bits |= child_bit;
        } else if (tree.nchild[cn] == 0) {
            settled_bits |= child_bit;
            if (child_accepted) accepted_bits |= child_bit;
        } else if (a.lazy && !(w_child > 0.0)) {
            // A child of weight 0 can never be accepted, passes weight 0 to its whole subtree
            // and never provides a bonus distribution: its task (and its subtree's) is not
            // queued, its rows are never read; the whole subtree counts as rejected.
            const int hi = tree.rank[cn], lo = tree.sub_lo[cn];
            const unsigned long long upto = (hi >= 63) ? ~0ull : ((1ull << (hi + 1)) - 1ull);
            settled_bits |= upto & ~((1ull << lo) - 1ull);
        }
        // Traversal: the child's own task is needed unless its weight is 0 (see above)
        const bool run_child = METHOD == MPV_METHOD_TRAVERSAL && !redone && tree.nchild[cn] > 0 && (w_child > 0.0 || !a.lazy);
        const bool first_to_run = run_child && own_child < 0;
        if (first_to_run) {
            // kept for this workgroup if it is the last thing this task finds out and nobody is idle
            own_child = j;
            own_given = (idle_seen || j < k - 1 || child_ahead) && !(split_here && j == 0);
        }
        // One more sweep to go at most: time to ask for the next task, unless this workgroup
        // already knows what it will run next (a child's task).
        if (j == k - 1 && !asked && (own_child < 0 || own_given) &&
            !(METHOD == MPV_METHOD_SPECINFER && a.lazy && child_accepted && tree.nchild[cn] > 0)) {
            if (threadIdx.x == 0) request_task(ws);
            asked = true;
        }
        if (threadIdx.x == 0 && !redone) {
            if (METHOD == MPV_METHOD_TRAVERSAL) {
                if (tree.nchild[cn] == 0) {
                    st_shared_f64(&ws.atest[bc], w_child);           // leaves are tested as they are
                } else {
                    __hip_atomic_store(reinterpret_cast<unsigned long long*>(&ws.a0[bc]),
                                       static_cast<unsigned long long>(__double_as_longlong(w_child)),
                                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    // The first child that needs a task is kept for this workgroup (run next,
                    // no queue) unless some workgroup is idle; every other one is queued now,
                    // while this task goes on with the sweeps that follow.
                    if (run_child && (!first_to_run || own_given) && !child_ahead) {
                        wait_memory();                    // its starting weight has been written
                        append_task(tree, ws, tree.cls[cn], b * a.N + cn);
                    }
                }
            } else {
                st_shared_f64(&ws.atest[bc], w_child);
                if (a.estimate && a.walk == 3) {
                    // App. D, SpecTr Branching: p_res(x), p_res = norm (p - rho* q)_+ (see the search above)
                    const double r = fmax(px - sp_rho * qx, 0.0);
                    st_shared_f64(&ws.aux[bc], sp_W > 0.0 ? fmin(r / sp_W, 1.0) : px);
                }
            }
            if (a.dbg_edge) {
                a.dbg_edge[bc * 2] = static_cast<float>(px);
                a.dbg_edge[bc * 2 + 1] = static_cast<float>(qx);
            }
        }

        // Where the tree branches and no workgroup is to spare, the first child's subtree is
        // explored first: most walks end there, and then nothing else of this node is needed.
        if (split_here && j == 0 && run_child) {
            paused = true;
            break;
        }

        if (METHOD == MPV_METHOD_SPECINFER && a.walk >= 2 && !a.estimate && threadIdx.x == 0 &&
            fabs(w_child - static_cast<double>(ch_u[j])) < 1e-6)
            atomicAdd(&a.counters[MPV_COUNTER_NEAR_TIE_ACCEPT], 1u);     // (the other rules count these in their walk)
        // SpecInfer moves into the first child it accepts: later children and this node's
        // residual are not needed (the same in every lane: no lane is left behind)
        if (METHOD == MPV_METHOD_SPECINFER && a.lazy && child_accepted) {
            next_node = cn;
            break;
        }
        // NSS: nothing else to find out here
        if (METHOD == MPV_METHOD_SPECINFER && a.walk == 1) continue;
        // Naive (App. B, Alg. 2) tests the first child only; the token then drawn comes from (p - q)_+
        if (METHOD == MPV_METHOD_SPECINFER && a.walk == 2 && !a.estimate) {
            c = 1.0;
            break;
        }
        // SpecTr tests every child against the same p; its residual is formed once, by the draw
        if (METHOD == MPV_METHOD_SPECINFER && a.walk == 3) {
            c = sp_rho;
            continue;
        }

        // ---- the child (SpecInfer) or its whole subtree (Traversal) is rejected:
        //      P <- norm (a P - q)_+ ,  i.e.  c <- c + W/a ,  W <- W(c)
        if (METHOD == MPV_METHOD_TRAVERSAL && !(wa > 0.0)) continue;   // (0*P - q)_+ = 0: nothing changes
        const double c2 = uniform_f64(c + W / wa);
        const ResidualConsts rc = residual_consts(rt.A, rd.A, c2);
        const double scale = uniform_f64(rc.scale);
        ResidualMassRawF<E> f;
        f.init();
        f.k32 = k32; f.nAt = rc.nAt; f.nAd = rc.nAd; f.rho = uniform_f32(rc.rho);
        pair.replay(f);
        const double lane_mass = static_cast<double>(f.acc0) + static_cast<double>(f.acc1);
        const double W2 = uniform_f64(scale * block_sum<kTaskBlock>(lane_mass, scratch));
        if (W2 > 0.0) {
            if (METHOD == MPV_METHOD_TRAVERSAL) {
                const double S = (wa / W) * W2;
                wa = uniform_f64(S / (S + (1.0 - wa)));
            }
            c = c2;
            W = W2;
        } else {
            if (METHOD == MPV_METHOD_TRAVERSAL) wa = (wa >= 1.0) ? 1.0 : 0.0;
            if (threadIdx.x == 0) atomicAdd(&a.counters[MPV_COUNTER_ZERO_MASS], 1u);
        }
        if (METHOD == MPV_METHOD_SPECINFER && a.walk == 2) {
            // Naive, estimate (App. D, Naive Branching): p_res(x_i) for every child, p_res = norm (p - q)_+
            // (now c = 1 and W = its mass; p itself if the mass was zero: c = 0, W = 1)
            for (int i = 0; i < k; ++i) {
                const int ci = tree.child_list[tree.child_off[n] + i];
                const int xi = ch_tok[i];
                double r = 0.0;
                if (xi >= 0 && xi < V)
                    r = fmax(exp2(static_cast<double>(ch_zt[i]) * kd - rt.A) - c * exp2(static_cast<double>(ch_zd[i]) * kd - rd.A), 0.0) / W;
                else if (i > 0 && threadIdx.x == 0)
                    atomicAdd(&a.counters[MPV_COUNTER_BAD_TOKEN], 1u);
                if (threadIdx.x == 0) {
                    st_shared_f64(&ws.aux[static_cast<size_t>(b) * a.N + ci], r);
                    if (i > 0) st_shared_f64(&ws.atest[static_cast<size_t>(b) * a.N + ci], 0.0);   // never tested
                }
                settled_bits |= 1ull << tree.rank[ci];
            }
            break;
        }
    }

    if (paused) {
        // nothing is settled yet; the first child's task is run next by this workgroup
        own_task = b * a.N + tree.child_list[tree.child_off[n]];
        if (threadIdx.x == 0) {
            (void)atomicAdd(&ws.qctl[0], 1);
            wait_memory();                            // counted (and the child's weight written) before this task counts as finished
            atomicAdd(&ws.qctl[1], 1);
        }
        continue;
    }
    __shared__ int sh_push_sample, sh_settled, sh_resume;
    if (threadIdx.x == 0) {
        st_shared_f64(&ws.At[bn], rt.A);
        st_shared_f64(&ws.Ad[bn], rd.A);
        st_shared_f64(&ws.cfin[bn], c);
        if (METHOD == MPV_METHOD_TRAVERSAL && n != 0) st_shared_f64(&ws.atest[bn], wa);
        bool push_sample, settled_tree = false, resume = false;
        if (METHOD == MPV_METHOD_SPECINFER && a.lazy) {
            // the walk ends here (no child accepted) or in the accepted leaf
            push_sample = next_node < 0 || tree.nchild[next_node] == 0;
            if (a.walk) st_relaxed(&ws.cur[b], next_node >= 0 ? next_node : n);     // where the next token is drawn
            wait_memory();                            // results written through before anything else is started
        } else {
            // Announce the outcomes settled here, then see whether the tree's outcome is settled:
            //   only what is needed: in postorder, the first node that is not known to be
            //     rejected is known (then it is the accepted one: the walk stops there);
            //   everything: every node is known.
            // `acc` is written before `known`, so the acc bits of known nodes are final.  Of
            // the tasks that see a settled tree, the first to flip `decided` starts the sampling.
            if (METHOD == MPV_METHOD_TRAVERSAL && n != 0) {
                const unsigned long long own = 1ull << tree.rank[n];
                settled_bits |= own;
                if (static_cast<double>(sh_un) < wa) accepted_bits |= own;
            }
            wait_memory();                            // results written through before they are announced
            if (accepted_bits) {
                (void)atomicOr(&ws.acc[b], accepted_bits);
                wait_memory();
            }
            const unsigned long long known_before = atomicOr(&ws.known[b], settled_bits);
            const unsigned long long known = known_before | settled_bits;
            wait_memory();
            const unsigned long long acc = ld_relaxed(&ws.acc[b]);
            const int decided_before = ld_relaxed(&ws.decided[b]);      // issued with the load above: one round trip
            bool settled;
            if (a.lazy) {
                const unsigned long long open = ~(known & ~acc);          // not known to be rejected
                const int first = __ffsll(static_cast<long long>(open)) - 1;   // the root's bit is always set
                settled = ((known >> first) & 1ull) != 0ull;
            } else {
                const unsigned long long all = (a.N >= 64) ? ~0ull : ((1ull << a.N) - 1ull);
                settled = known == all;
            }
            push_sample = settled && decided_before == 0 && atomicCAS(&ws.decided[b], 0, 1) == 0;
            // only what is needed: once a tree is settled (here or by another task) the rest of
            // its node tasks are pointless
            settled_tree = a.lazy && (settled || decided_before != 0);
            // The subtree that was explored first has just turned out to be rejected as a whole
            // (this task supplied its last missing outcome): time for the rest of the node
            // where the tree branches.
            if (METHOD == MPV_METHOD_TRAVERSAL && a.lazy && q.split_node >= 0 && !settled_tree &&
                ((q.split_mask >> tree.rank[n]) & 1ull) != 0ull) {          // this node lies in that subtree
                const unsigned long long m = q.split_mask;
                resume = (known & m) == m && (known_before & m) != m && (acc & m) == 0ull;
            }
        }
        sh_push_sample = push_sample ? 1 : 0;
        sh_settled = settled_tree ? 1 : 0;
        sh_resume = resume ? 1 : 0;
    }
    __syncthreads();
    // What follows from this task.  One task is run by this workgroup itself, next (no queue,
    // no waiting): the sampling if this task settled the tree, else the first child that needs
    // its own task (Traversal) or the accepted child (SpecInfer).  The other children are queued.
    if (sh_push_sample) {
        own_task = a.B * a.N + b;
    } else if (sh_resume) {
        own_task = a.B * a.N + a.B + b;
    } else if (METHOD == MPV_METHOD_TRAVERSAL) {
        if (own_child >= 0 && !own_given && !sh_settled) own_task = b * a.N + tree.child_list[tree.child_off[n] + own_child];
    } else if (a.lazy && next_node >= 0 && tree.nchild[next_node] > 0) {
        own_task = b * a.N + next_node;
    }
    if (threadIdx.x == 0) {
        if (own_task >= 0) {
            (void)atomicAdd(&ws.qctl[0], 1);
            wait_memory();
        }
        // (cannot happen: a task that settles the tree or completes a subtree has no child left to run)
        if (METHOD == MPV_METHOD_TRAVERSAL && own_child >= 0 && !own_given && !sh_settled && (sh_push_sample || sh_resume)) {
            const int cn = tree.child_list[tree.child_off[n] + own_child];
            append_task(tree, ws, tree.cls[cn], b * a.N + cn);
        }
    }
    __syncthreads();                                  // every new task has been counted
    if (threadIdx.x == 0) atomicAdd(&ws.qctl[1], 1);
    }   // task loop
}

// ------------------------------------------------------------------ walk
//
// The uniform-dependent part of SpecInfer and Traversal, run by the first wave of the sampling
// workgroup: lane n compares u[n] with the probability node n is tested with
// (which does not depend on the uniforms), the 64 outcomes become a bit mask, and
// the walk itself is a few scalar steps over that mask.
//   SpecInfer (Sec. 3.2 walk + App. B Alg. 4): from the root, move to the first
//     accepted child in list order; stop where no child is accepted.
//   Traversal: nodes are tested in depth-first post-order; the first accepted one
//     wins, the root is accepted unconditionally.
// Returns the stopping node (the same value in every lane) and writes the path.
// accepted length and path of a walk that ended in `stop` (one lane)
__device__ __forceinline__ void write_path(const TreeDesc& tree, const Args& a, int b, int stop) {
    const size_t base = static_cast<size_t>(b) * a.N;
    const int len = tree.depth[stop];
    a.accept_len[b] = len;
    int32_t* pn = a.path_nodes + static_cast<size_t>(b) * a.max_depth;
    int32_t* pt = a.path_tokens + static_cast<size_t>(b) * a.max_depth;
    for (int i = len; i < a.max_depth; ++i) { pn[i] = -1; pt[i] = -1; }
    for (int n = stop, i = len - 1; n > 0; n = tree.parent[n], --i) {
        pn[i] = n;
        pt[i] = a.tokens[base + n];
    }
}

template <int METHOD>
__device__ __forceinline__ int walk_wave(const TreeDesc& tree, const Workspace& ws, const Args& a, int b) {
    const int lane = threadIdx.x & (kWave - 1);
    const size_t base = static_cast<size_t>(b) * a.N;
    bool acc = false, near = false;
    if (lane > 0 && lane < a.N) {
        const double at = ld_shared_f64(&ws.atest[base + lane]);
        const double uu = static_cast<double>(a.uniforms[base + lane]);
        acc = uu < at;
        near = fabs(at - uu) < 1e-6;
        if (a.dbg_accept) a.dbg_accept[base + lane] = static_cast<float>(at);
    }
    if (lane == 0 && a.dbg_accept) a.dbg_accept[base] = 1.f;
    const unsigned long long accm = __ballot(acc);
    const unsigned long long nearm = __ballot(near);
    unsigned long long tested = 0ull;
    int stop = 0;
    if (METHOD == MPV_METHOD_SPECINFER) {
        int n = 0;
        for (;;) {
            int next = -1;
            const int k = tree.nchild[n], off = tree.child_off[n];
            for (int j = 0; j < k; ++j) {
                const int cn = tree.child_list[off + j];
                tested |= 1ull << cn;
                if ((accm >> cn) & 1ull) { next = cn; break; }
            }
            if (next < 0) break;
            n = next;
        }
        stop = n;
    } else {
        for (int i = 0; i + 1 < a.N; ++i) {
            const int n = tree.postorder[i];
            tested |= 1ull << n;
            if ((accm >> n) & 1ull) { stop = n; break; }
        }
    }
    if (lane == 0) {
        write_path(tree, a, b, stop);
        const int nn = __popcll(nearm & tested);
        if (nn) atomicAdd(&a.counters[MPV_COUNTER_NEAR_TIE_ACCEPT], static_cast<unsigned>(nn));
    }
    return stop;
}

// ------------------------------------------------------------------ expected block efficiency
//
// Sec. 5, Eq. 1-3: E[tau + 1 | tree] = sum over nodes of P(the node lies on the accepted path).
// Lane n looks after node n.  Top-down rules: the probability of moving from a node to its
// child is put together from the per-child results the node tasks left (App. D):
//   SpecInfer  a_j prod_{l<j} (1 - a_l), a_l the probability sibling l is tested with;
//   NSS        p(x_j) if no earlier sibling carries the same token (a drawn token leads to the
//              first sibling that carries it), else 0;
//   Naive      [j = 1] a_1 + (1 - a_1) p_res(x_j) [first carrier of x_j];
//   SpecTr     a_j prod_{l<j} (1 - a_l) + p_res(x_j) prod_l (1 - a_l) [first carrier of x_j];
// and a node's reach probability is the product along its path from the root.  Traversal: nodes
// are tested in postorder, each after everything before it was rejected, so the node at position
// r is the accepted one with a_r prod_{r'<r} (1 - a_r'), and a node is on the accepted path iff
// the accepted node is in its subtree.
template <int METHOD>
__device__ __forceinline__ void estimate_wave(const TreeDesc& tree, const Workspace& ws, const Args& a, int b) {
    __shared__ double sh_v[MPV_MAX_NODES], sh_w[MPV_MAX_NODES];
    const int n = threadIdx.x & (kWave - 1);
    const size_t base = static_cast<size_t>(b) * a.N;
    const bool live = n < a.N;
    double reach = 0.0;
    if (METHOD == MPV_METHOD_TRAVERSAL) {
        // sh_v[r]: test probability of the node at postorder position r (the root, last, is accepted)
        if (live) {
            const int node = tree.postorder[n];
            sh_v[n] = (node == 0) ? 1.0 : ld_shared_f64(&ws.atest[base + node]);
        }
        __builtin_amdgcn_wave_barrier();
        if (live) {
            double none_before = 1.0;
            for (int r = 0; r < n; ++r) none_before *= 1.0 - sh_v[r];
            sh_w[n] = sh_v[n] * none_before;          // the node at position n is the accepted one
        }
        __builtin_amdgcn_wave_barrier();
        if (live) {
            if (n == 0) reach = 1.0;
            else for (int r = tree.sub_lo[n]; r <= tree.rank[n]; ++r) reach += sh_w[r];
        }
    } else {
        if (live) {
            sh_v[n] = (n == 0) ? 1.0 : ld_shared_f64(&ws.atest[base + n]);
            sh_w[n] = (n == 0 || a.walk < 2) ? 0.0 : ld_shared_f64(&ws.aux[base + n]);
        }
        __builtin_amdgcn_wave_barrier();
        double step = 1.0;                            // from the parent to this node
        if (live && n > 0) {
            const int par = tree.parent[n], off = tree.child_off[par], k = tree.nchild[par];
            const int x = a.tokens[base + n];
            double none_before = 1.0, none_at_all = 1.0;
            bool first_carrier = true;
            int j = 0;
            for (int l = 0; l < k; ++l) {
                const int sib = tree.child_list[off + l];
                if (sib == n) j = l;
                if (sib < n) {                        // list order is node order
                    none_before *= 1.0 - sh_v[sib];
                    if (a.tokens[base + sib] == x) first_carrier = false;
                }
                none_at_all *= 1.0 - sh_v[sib];
            }
            if (a.walk == 0) step = sh_v[n] * none_before;
            else if (a.walk == 1) step = first_carrier ? sh_v[n] : 0.0;
            else if (a.walk == 2) {
                const double a1 = sh_v[tree.child_list[off]];
                step = (j == 0 ? a1 : 0.0) + (first_carrier ? (1.0 - a1) * sh_w[n] : 0.0);
            } else {
                step = sh_v[n] * none_before + (first_carrier ? sh_w[n] * none_at_all : 0.0);
            }
        }
        __builtin_amdgcn_wave_barrier();              // everybody has read sh_v / sh_w
        if (live) sh_v[n] = step;
        __builtin_amdgcn_wave_barrier();
        if (live) {
            reach = 1.0;
            for (int m = n; m > 0; m = tree.parent[m]) reach *= sh_v[m];
        }
    }
    if (live && a.reach_prob) a.reach_prob[base + n] = static_cast<float>(reach);
    const double total = wave_sum(live ? reach : 0.0);
    if (n == 0 && a.expected) a.expected[b] = static_cast<float>(total);
}

// ------------------------------------------------------------------ bonus sample

// r_v = (p_v - c q_v)_+ up to the common factor 2^-At_lo, for the VEC elements a lane
// owns in wave tile `tile` (elements [tile * 64 * VEC, (tile + 1) * 64 * VEC); zero beyond V).
// A vector load when the rows are 16-byte aligned, element loads otherwise.
template <class E>
struct ResidualTile {
    static constexpr int PER_LANE = E::VEC;
    static constexpr int TILE = kWave * E::VEC;
    const typename E::T* zt;
    const typename E::T* zd;
    int V;
    bool aligned, use_d;
    float k32, nAt, nAd, rho;

    __device__ __forceinline__ void load(int tile, int lane, float (&r)[PER_LANE]) const {
        const int e0 = tile * TILE + lane * PER_LANE;
        if (aligned && e0 + PER_LANE <= V) {
            float t[PER_LANE], d[PER_LANE];
            E::load_vec(zt + e0, t);
            if (use_d) E::load_vec(zd + e0, d);
#pragma unroll
            for (int i = 0; i < PER_LANE; ++i) r[i] = term(t[i], use_d ? d[i] : 0.f);
        } else {
#pragma unroll
            for (int i = 0; i < PER_LANE; ++i) {
                const int e = e0 + i;
                r[i] = (e < V) ? term(E::load_one(zt + e), use_d ? E::load_one(zd + e) : 0.f) : 0.f;
            }
        }
    }
    __device__ __forceinline__ float term(float t, float d) const {
        const float et = fast_exp2(fmaf(t, k32, nAt));
        if (!use_d) return et;
        const float ed = fast_exp2(fmaf(d, k32, nAd));
        return fmaxf(fmaf(-rho, ed, et), 0.f);
    }
};


// tile_sum: kMaxTiles floats of LDS; scratch: 2 doubles per wave.  Everything it reads from
// the workspace was written by node tasks of this launch (see st_shared_f64).
template <class E, int METHOD>
__device__ __forceinline__ int sample_task(const TreeDesc& tree, const Workspace& ws, const Args& a, int b,
                           float* tile_sum, double* scratch) {
    using T = typename E::T;
    constexpr int NW = kSampleBlock / kWave;
    constexpr int PER_LANE = ResidualTile<E>::PER_LANE;
    constexpr int TILE = ResidualTile<E>::TILE;
    __shared__ int sh_tile;
    __shared__ double sh_before, sh_total, sh_target;

    __shared__ int sh_stop, sh_next;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    if (wave == 0) {
        // where the token is drawn: the node the rule stops in, or the node a token-following
        // walk has reached
        const int stop = a.walk ? ld_relaxed(&ws.cur[b]) : walk_wave<METHOD>(tree, ws, a, b);
        if (lane == 0) { sh_stop = stop; sh_next = -1; }
    }
    __syncthreads();
    const int n = __builtin_amdgcn_readfirstlane(sh_stop);
    const size_t bn = static_cast<size_t>(b) * a.N + n;
    const T* zt = static_cast<const T*>(a.zt) + bn * a.V;
    const T* zd = static_cast<const T*>(a.zd) + bn * a.V;
    const int V = a.V;
    const int ntiles = (V + TILE - 1) / TILE;

    double At, Ad = 0.0, c = 0.0;
    if (tree.nchild[n] == 0 || a.walk == 1) {
        // a leaf (its target row has not been touched yet) or an NSS draw: from p itself
        RowStatsF<E> f;
        f.t.init(); f.k32 = a.k32;
        sweep_row<E, kSampleBlock, 4 * kTaskUnroll>(zt, V, f);     // alone on its compute unit: many loads in flight
        OnlineLse none; none.init();
        RowStat rt, rd;
        finish_stats2<kSampleBlock>(f.t, none, rt, rd, scratch);
        At = rt.A;
        if (threadIdx.x == 0) ws.At[bn] = rt.A;
    } else {
        At = ld_shared_f64(&ws.At[bn]);
        Ad = ld_shared_f64(&ws.Ad[bn]);
        c = ld_shared_f64(&ws.cfin[bn]);
    }

    ResidualTile<E> rt_;
    rt_.zt = zt; rt_.zd = zd; rt_.V = V;
    rt_.aligned = ((reinterpret_cast<uintptr_t>(zt) & 15u) == 0);
    rt_.use_d = (c > 0.0);
    rt_.k32 = a.k32;
    if (rt_.use_d) {
        const ResidualConsts rc = residual_consts(At, Ad, c);
        rt_.nAt = rc.nAt; rt_.nAd = rc.nAd; rt_.rho = rc.rho;
    } else {
        rt_.nAt = -static_cast<float>(At); rt_.nAd = 0.f; rt_.rho = 0.f;
    }

    // ---- pass 1: mass of every wave tile, in vocabulary order
    {
        // Whole, aligned tiles are taken U at a time per wave with all their loads issued
        // before the first use: one workgroup per compute unit hides memory latency only by
        // the loads each wave keeps in flight.
        int t_next = wave;
        constexpr int U = 8;
        const int whole = rt_.aligned ? V / TILE : 0;
        for (; t_next + (U - 1) * NW < whole; t_next += U * NW) {
            uint4 qt[U], qd[U];
#pragma unroll
            for (int j = 0; j < U; ++j) {
                const int e0 = (t_next + j * NW) * TILE + lane * PER_LANE;
                qt[j] = load_raw(zt + e0);
                if (rt_.use_d) qd[j] = load_raw(zd + e0);
            }
            float s[U];
#pragma unroll
            for (int j = 0; j < U; ++j) {
                float tv[PER_LANE], dv[PER_LANE];
                E::unpack(qt[j], tv);
                if (rt_.use_d) E::unpack(qd[j], dv);
                float ls = 0.f;                       // same order of additions as pass 2
#pragma unroll
                for (int i = 0; i < PER_LANE; ++i) ls += rt_.term(tv[i], rt_.use_d ? dv[i] : 0.f);
                s[j] = ls;
            }
#pragma unroll
            for (int j = 0; j < U; ++j) s[j] = wave_sum_f32(s[j]);
            if (lane == 0) {
#pragma unroll
                for (int j = 0; j < U; ++j) tile_sum[t_next + j * NW] = s[j];
            }
        }
        for (int t = t_next; t < ntiles; t += NW) {
            float r[PER_LANE];
            rt_.load(t, lane, r);
            float ls = 0.f;
#pragma unroll
            for (int i = 0; i < PER_LANE; ++i) ls += r[i];
            const float w = wave_sum_f32(ls);
            if (lane == 0) tile_sum[t] = w;
        }
    }
    __syncthreads();

    // ---- locate the tile that contains u * R (wave 0; each lane owns a run of tiles)
    if (wave == 0) {
        const int per = (ntiles + kWave - 1) / kWave;
        const int t0 = lane * per, t1 = min(t0 + per, ntiles);
        double run = 0.0;
        for (int t = t0; t < t1; ++t) run += tile_sum[t];
        const double incl = wave_inclusive_scan(run);
        const double total = __shfl(incl, kWave - 1, kWave);
        const float u_draw = a.walk ? a.draw_uniforms[bn] : a.uniforms[static_cast<size_t>(b) * a.N];
        const double target = static_cast<double>(u_draw) * total;
        const unsigned long long hit = __ballot(incl > target && run > 0.0);
        int owner = hit ? (__ffsll(static_cast<long long>(hit)) - 1) : -1;
        if (owner < 0) {           // rounding only: last lane that has mass
            const unsigned long long any = __ballot(run > 0.0);
            owner = any ? (63 - __clzll(static_cast<long long>(any))) : 0;
        }
        if (lane == owner) {
            double acc = incl - run;
            int found = -1, last_mass = t0;
            double before = acc;
            for (int t = t0; t < t1; ++t) {
                const double ts = tile_sum[t];
                if (ts > 0.0) last_mass = t;
                if (found < 0 && acc + ts > target && ts > 0.0) { found = t; before = acc; }
                acc += ts;
            }
            if (found < 0) {       // rounding only: last tile of the run that has mass
                found = last_mass;
                before = incl - run;
                for (int t = t0; t < last_mass; ++t) before += tile_sum[t];
            }
            sh_tile = found;
            sh_before = before;
            sh_total = total;
            sh_target = target;
        }
    }
    __syncthreads();

    // ---- pass 2: inside that tile (wave 0)
    if (wave == 0) {
        const int t = sh_tile;
        const double rem = sh_target - sh_before;       // mass to cover inside the tile
        float r[PER_LANE];
        rt_.load(t, lane, r);
        float ls = 0.f;
#pragma unroll
        for (int i = 0; i < PER_LANE; ++i) ls += r[i];
        const double lsd = static_cast<double>(ls);
        const double incl = wave_inclusive_scan(lsd);
        const unsigned long long hit = __ballot(incl > rem && ls > 0.f);
        int owner = hit ? (__ffsll(static_cast<long long>(hit)) - 1) : -1;
        if (owner < 0) {
            const unsigned long long any = __ballot(ls > 0.f);
            owner = any ? (63 - __clzll(static_cast<long long>(any))) : 0;
        }
        if (lane == owner) {
            double acc = incl - lsd;
            int found = -1, last_mass = 0;
            double lo = acc, hi = acc;
            for (int i = 0; i < PER_LANE; ++i) {
                const double ri = static_cast<double>(r[i]);
                if (ri > 0.0) last_mass = i;
                if (found < 0 && ri > 0.0 && acc + ri > rem) { found = i; lo = acc; hi = acc + ri; }
                acc += ri;
            }
            if (found < 0) { found = last_mass; lo = rem; hi = rem; }
            int tok = t * TILE + lane * PER_LANE + found;
            if (tok >= V) tok = V - 1;
            a.bonus[b] = tok;
            sh_tile = tok;                            // (the tile number is no longer needed)
            const double gap = fmin(fabs(rem - lo), fabs(hi - rem));
            if (gap < 1e-6 * sh_total) atomicAdd(&a.counters[MPV_COUNTER_NEAR_TIE_BONUS], 1u);
        }
        if (a.walk) {
            // Sec. 3.2: if the drawn token is a child's token the walk moves to that child (the
            // first such child in list order), otherwise it ends here
            __builtin_amdgcn_wave_barrier();
            const int tok = *reinterpret_cast<volatile int*>(&sh_tile);
            const int k = tree.nchild[n];
            bool same = false;
            if (lane < k) same = a.tokens[static_cast<size_t>(b) * a.N + tree.child_list[tree.child_off[n] + lane]] == tok;
            const unsigned long long m = __ballot(same);
            if (m) {
                const int to = tree.child_list[tree.child_off[n] + __ffsll(static_cast<long long>(m)) - 1];
                if (lane == 0) {
                    st_relaxed(&ws.cur[b], to);
                    // Naive and SpecTr test children of an inner node before they draw there; NSS and leaves draw at once
                    sh_next = (a.walk >= 2 && tree.nchild[to] > 0) ? b * a.N + to : a.B * a.N + b;
                }
            } else {
                if (lane == 0) write_path(tree, a, b, n);
                if (a.dbg_accept && lane < a.N)
                    a.dbg_accept[static_cast<size_t>(b) * a.N + lane] =
                        lane == 0 ? 1.f : static_cast<float>(ld_shared_f64(&ws.atest[static_cast<size_t>(b) * a.N + lane]));
            }
        }
    }

    // ---- optional: the normalised distribution itself
    if (a.dbg_resid) {
        const double inv = 1.0 / sh_total;
        float* out = a.dbg_resid + static_cast<size_t>(b) * V;
        for (int t = wave; t < ntiles; t += NW) {
            float r[PER_LANE];
            rt_.load(t, lane, r);
#pragma unroll
            for (int i = 0; i < PER_LANE; ++i) {
                const int e = t * TILE + lane * PER_LANE + i;
                if (e < V) out[e] = static_cast<float>(static_cast<double>(r[i]) * inv);
            }
        }
    }
    __syncthreads();
    return sh_next;
}

// ------------------------------------------------------------------ stand-alone row statistics

template <class E>
__global__ __launch_bounds__(kTaskBlock) void row_stats_kernel(const typename E::T* z, int64_t rows, int V,
                                                              float k32, float* out) {
    __shared__ double scratch[2 * (kTaskBlock / kWave)];
    const int64_t r = blockIdx.x;
    RowStatsF<E> f;
    f.t.init(); f.k32 = k32;
    sweep_row<E, kTaskBlock, kTaskUnroll>(z + r * V, V, f);
    OnlineLse none; none.init();
    RowStat rt, rd;
    finish_stats2<kTaskBlock>(f.t, none, rt, rd, scratch);
    if (threadIdx.x == 0) {
        out[2 * r] = rt.m;
        // ln sum exp((z-m)/T) = ln2 * (A - m*k32)
        out[2 * r + 1] = static_cast<float>(0.6931471805599453 * (rt.A - static_cast<double>(rt.m) * static_cast<double>(k32)));
    }
}

// Debug statistics [B,N,4] from the workspace (internal nodes, stopping leaves) --
// rows the path never touched are computed here.
template <class E>
__global__ __launch_bounds__(kTaskBlock) void debug_stats_kernel(TreeDesc tree, Args a) {
    using T = typename E::T;
    __shared__ double scratch[2 * (kTaskBlock / kWave)];
    const int64_t bn = blockIdx.x;
    const int n = static_cast<int>(bn % a.N);
    const T* zt = static_cast<const T*>(a.zt) + bn * a.V;
    const T* zd = static_cast<const T*>(a.zd) + bn * a.V;
    const bool leaf = tree.nchild[n] == 0;
    RowStat rt, rd;
    if (leaf) {
        RowStatsF<E> f;
        f.t.init(); f.k32 = a.k32;
        sweep_row<E, kTaskBlock, kTaskUnroll>(zt, a.V, f);
        OnlineLse none; none.init();
        finish_stats2<kTaskBlock>(f.t, none, rt, rd, scratch);
    } else {
        PairStatsF<E, kTaskBlock, kTaskUnroll> f;
        f.t.init(); f.d.init(); f.k32 = a.k32;
        sweep_pair<E, kTaskBlock, kTaskUnroll>(zt, zd, a.V, f);
        finish_stats2<kTaskBlock>(f.t, f.d, rt, rd, scratch);
    }
    if (threadIdx.x == 0) {
        const double kd = static_cast<double>(a.k32);
        float* o = a.dbg_stats + bn * 4;
        o[0] = rt.m;
        o[1] = static_cast<float>(0.6931471805599453 * (rt.A - static_cast<double>(rt.m) * kd));
        o[2] = leaf ? NAN : rd.m;
        o[3] = leaf ? NAN : static_cast<float>(0.6931471805599453 * (rd.A - static_cast<double>(rd.m) * kd));
    }
}

// ------------------------------------------------------------------ uniforms

__global__ void fill_uniforms_kernel(uint64_t seed, int64_t count, float* out) {
    const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i >= count) return;
    uint64_t z = seed + static_cast<uint64_t>(i + 1) * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    z = z ^ (z >> 31);
    out[i] = static_cast<float>(z >> 40) * (1.0f / 16777216.0f);
}

// ------------------------------------------------------------------ host side

thread_local int g_last_hip_error = 0;

static bool hip_ok(hipError_t e) {
    if (e == hipSuccess) return true;
    g_last_hip_error = static_cast<int>(e);
    return false;
}

// Optional per-launch timing: when enabled, every kernel launched by mpv_verify carries a pair
// of hipEvents that the runtime stamps with the start and the end of that dispatch itself
// (hipExtLaunchKernelGGL): no extra packet goes into the stream, the launches stay back to back.
struct LaunchTimer {
    bool enabled = false;
    int capacity = 0, used = 0;
    hipEvent_t* start = nullptr;
    hipEvent_t* stop = nullptr;
    int32_t* kernel = nullptr;
};
static LaunchTimer g_timer;

template <typename... Params, typename... Args>
static void launch(int kernel_id, void (*kernel)(Params...), dim3 grid, dim3 block, hipStream_t s, Args... args) {
    if (g_timer.enabled && g_timer.used < g_timer.capacity) {
        const int slot = g_timer.used++;
        g_timer.kernel[slot] = kernel_id;
        hipExtLaunchKernelGGL(kernel, grid, block, 0, s, g_timer.start[slot], g_timer.stop[slot], 0,
                              static_cast<Params>(args)...);
    } else {
        hipLaunchKernelGGL(kernel, grid, block, 0, s, static_cast<Params>(args)...);
    }
}

struct Plan {
    TreeDesc tree;
    int max_tree_depth;
    int n_internal;
    int nclass;
};

static int validate(const mpv_problem* p, Plan* plan) {
    if (!p) return MPV_ERR_NULL;
    if (p->B < 0 || p->N < 1 || p->V < 1) return MPV_ERR_BAD_SHAPE;
    if (p->N > MPV_MAX_NODES || p->V > MPV_MAX_VOCAB) return MPV_ERR_UNSUPPORTED;
    // task numbers (tree * N + node, and two more per tree) are 32-bit
    if (static_cast<int64_t>(p->B) * (p->N + 2) > (1ll << 30)) return MPV_ERR_UNSUPPORTED;
    if (p->method < MPV_METHOD_SPECINFER || p->method > MPV_METHOD_SPECTR) return MPV_ERR_BAD_METHOD;
    if (p->logit_dtype != MPV_DTYPE_F32 && p->logit_dtype != MPV_DTYPE_BF16) return MPV_ERR_BAD_DTYPE;
    if (!(p->temperature > 0.0f) || !isfinite(p->temperature)) return MPV_ERR_BAD_TEMPERATURE;
    if (!p->parent) return MPV_ERR_NULL;
    if (p->parent[0] != -1) return MPV_ERR_BAD_TREE;
    TreeDesc& t = plan->tree;
    memset(&t, 0, sizeof(t));
    t.N = p->N;
    t.parent[0] = -1;
    int nch[MPV_MAX_NODES] = {0};
    for (int n = 1; n < p->N; ++n) {
        const int par = p->parent[n];
        if (par < 0 || par >= n) return MPV_ERR_BAD_TREE;
        t.parent[n] = par;
        t.depth[n] = t.depth[par] + 1;
        ++nch[par];
    }
    int off = 0, maxd = 0, internal = 0;
    for (int n = 0; n < p->N; ++n) {
        if (nch[n] > MPV_MAX_CHILDREN) return MPV_ERR_UNSUPPORTED;
        t.nchild[n] = nch[n];
        t.child_off[n] = off;
        off += nch[n];
        if (t.depth[n] > maxd) maxd = t.depth[n];
        if (nch[n]) ++internal;
    }
    int fill[MPV_MAX_NODES] = {0};
    for (int n = 1; n < p->N; ++n) {
        const int par = t.parent[n];
        t.child_list[t.child_off[par] + fill[par]++] = n;
    }
    {   // depth-first post-order without recursion
        int next_child[MPV_MAX_NODES] = {0};
        int n = 0, out = 0;
        for (;;) {
            if (next_child[n] < t.nchild[n]) {
                n = t.child_list[t.child_off[n] + next_child[n]++];
                continue;
            }
            t.postorder[out++] = n;
            if (n == 0) break;
            n = t.parent[n];
        }
    }
    for (int r = 0; r < p->N; ++r) t.rank[t.postorder[r]] = r;
    for (int r = 0; r < p->N; ++r) {                  // children come before their parent
        const int n = t.postorder[r];
        t.sub_lo[n] = t.nchild[n] ? t.sub_lo[t.child_list[t.child_off[n]]] : r;
    }
    {   // priority classes: 0 from the root down to the first node that branches, 1 below it
        int branch = 0;
        while (t.nchild[branch] == 1) branch = t.child_list[t.child_off[branch]];
        for (int n = 0; n < p->N; ++n) t.cls[n] = (t.depth[n] <= t.depth[branch]) ? 0 : 1;
        plan->nclass = t.nchild[branch] ? 2 : 1;
    }
    plan->max_tree_depth = maxd;
    plan->n_internal = internal;
    if (p->max_depth < maxd) return MPV_ERR_BAD_SHAPE;
    return MPV_OK;
}

static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

static size_t carve(const mpv_problem* p, void* base, Workspace* ws) {
    const size_t bn = static_cast<size_t>(p->B) * p->N;
    size_t off = 0;
    char* b = static_cast<char*>(base);
    auto take = [&](size_t bytes) { void* q = b ? b + off : nullptr; off = align_up(off + bytes, 256); return q; };
    double* At = static_cast<double*>(take(bn * 8));
    double* Ad = static_cast<double*>(take(bn * 8));
    double* cf = static_cast<double*>(take(bn * 8));
    double* ax = static_cast<double*>(take(bn * 8));
    double* a0 = static_cast<double*>(take(bn * 8));
    double* at = static_cast<double*>(take(bn * 8));
    int32_t* qu = static_cast<int32_t*>(take(bn * 4));
    int32_t* qc = static_cast<int32_t*>(take((5 + 2 * kMaxClasses) * 4));
    int32_t* mb = static_cast<int32_t*>(take(kMaxWorkgroups * 4));
    unsigned long long* kn = static_cast<unsigned long long*>(take(static_cast<size_t>(p->B) * 8));
    unsigned long long* ac = static_cast<unsigned long long*>(take(static_cast<size_t>(p->B) * 8));
    int32_t* de = static_cast<int32_t*>(take(static_cast<size_t>(p->B) * 4));
    int32_t* cu = static_cast<int32_t*>(take(static_cast<size_t>(p->B) * 4));
    TreeDesc* tr = static_cast<TreeDesc*>(take(sizeof(TreeDesc)));
    if (ws) { ws->At = At; ws->Ad = Ad; ws->cfin = cf; ws->aux = ax; ws->a0 = a0; ws->atest = at; ws->queue = qu; ws->qctl = qc; ws->mailbox = mb; ws->known = kn; ws->acc = ac; ws->decided = de; ws->cur = cu; ws->tree = tr; }
    return off < 256 ? 256 : off;
}

static int compute_units() {
    static int cus = 0;
    if (cus == 0) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
            cus = n;
        else
            cus = 256;
    }
    return cus;
}

// Start-up spread of the persistent workgroups (Args::stagger_ticks): about the time one
// workgroup needs to read a row pair when every compute unit is reading (its share of
// ~6.3 TB/s), only for rows long enough to be kept on chip (short rows finish before it
// would matter).
static int32_t stagger_ticks(const mpv_problem* p) {
    const double pair_bytes = 2.0 * p->V * (p->logit_dtype == MPV_DTYPE_F32 ? 4 : 2);
    const double share_bytes_per_us = 6.3e6 / compute_units();
    const double us = pair_bytes / share_bytes_per_us;
    return (pair_bytes >= 400e3) ? static_cast<int32_t>(us * 100.0 / 8.0) : 0;
}

template <class E>
static int launch_all(const mpv_problem* p, const Plan& plan, const Workspace& ws, const Args& a, hipStream_t s) {
    TreeDesc tree = plan.tree;
    (void)hipGetLastError();    // a stale error left by the caller's own HIP calls is not ours
    // every register and LDS slot of a node task is populated whatever the row's alignment
    const bool full = (p->V - (E::VEC - 1)) / E::VEC >= (kRegVecs + kLdsVecs) * kTaskBlock;
    // Queue layout and initial tasks.  Computing only what is needed, both rules start from the
    // root: SpecInfer queues the accepted child, Traversal the children of positive weight.
    // Computing everything (debug outputs), SpecInfer's node tasks are independent and all
    // queued up front, nodes with many children (the long tasks) first.
    QueuePlan q;
    memset(&q, 0, sizeof(q));
    q.nclass = plan.nclass;
    int in_class[kMaxClasses] = {0};
    for (int n = 0; n < p->N; ++n)
        if (tree.nchild[n]) ++in_class[tree.cls[n]];
    for (int c = 0; c < q.nclass; ++c)
        q.off[c + 1] = q.off[c] + p->B * (in_class[c] + (c == 0 ? 1 : 0));     // class 0 also holds the sampling tasks
    int prequeued[kMaxClasses] = {0};
    for (int n = 0; n < p->N; ++n) q.init_slot[n] = -1;
    const bool all_up_front = (p->method != MPV_METHOD_TRAVERSAL && !a.lazy);
    for (int kk = MPV_MAX_CHILDREN; kk >= 1; --kk)
        for (int n = 0; n < p->N; ++n)
            if (tree.nchild[n] == kk && (all_up_front || n == 0) && (a.walk != 1 || !a.lazy))      // NSS verification has no node tasks
                q.init_slot[n] = prequeued[tree.cls[n]]++;
    for (int c = 0; c < q.nclass; ++c) {
        q.init_tail[c] = prequeued[c] * p->B;
        q.init_total += q.init_tail[c];
    }
    if (tree.nchild[0] == 0 || (a.walk == 1 && a.lazy)) {
        q.root_is_leaf = 1;
        q.init_tail[0] = p->B;
        q.init_total = p->B;
    }
    for (int c = 0; c <= q.nclass; ++c) tree.class_off[c] = q.off[c];
    const int tasks = q.off[q.nclass];
    // about one workgroup per compute unit (a node task fills one); fewer if there is less to do
    int wgs = tasks < compute_units() ? tasks : compute_units();
    if (wgs > kMaxWorkgroups) wgs = kMaxWorkgroups;
    q.workers = wgs;
    q.split_node = -1;
    if (p->method == MPV_METHOD_TRAVERSAL && a.lazy && p->B >= wgs) {
        int branch = 0;
        while (tree.nchild[branch] == 1) branch = tree.child_list[tree.child_off[branch]];
        if (tree.nchild[branch] >= 2) {
            const int first = tree.child_list[tree.child_off[branch]];
            if (tree.nchild[first] > 0) {
                const int hi = tree.rank[first], lo = tree.sub_lo[first];
                const unsigned long long upto = (hi >= 63) ? ~0ull : ((1ull << (hi + 1)) - 1ull);
                q.split_node = branch;
                q.split_mask = upto & ~((1ull << lo) - 1ull);
            }
        }
    }
    {
        const int threads = 256;
        const int blocks = (max(p->B, 64) + threads - 1) / threads;
        launch(MPV_KERNEL_INIT, init_kernel, dim3(blocks, p->N), dim3(threads), s, q, tree, ws, a);
    }
    if (tasks > 0) {
        const dim3 grid(static_cast<unsigned>(wgs)), block(kTaskBlock);
        if (a.estimate == 2) {
            if (full) launch(MPV_KERNEL_NODE_TASK, node_task_kernel<E, kKindAcceptance, true>, grid, block, s, q, ws, a);
            else launch(MPV_KERNEL_NODE_TASK, node_task_kernel<E, kKindAcceptance, false>, grid, block, s, q, ws, a);
        } else if (p->method != MPV_METHOD_TRAVERSAL) {      // NSS, Naive and SpecTr are variants of the top-down kernel
            if (full) launch(MPV_KERNEL_NODE_TASK, node_task_kernel<E, MPV_METHOD_SPECINFER, true>, grid, block, s, q, ws, a);
            else launch(MPV_KERNEL_NODE_TASK, node_task_kernel<E, MPV_METHOD_SPECINFER, false>, grid, block, s, q, ws, a);
        } else {
            if (full) launch(MPV_KERNEL_NODE_TASK, node_task_kernel<E, MPV_METHOD_TRAVERSAL, true>, grid, block, s, q, ws, a);
            else launch(MPV_KERNEL_NODE_TASK, node_task_kernel<E, MPV_METHOD_TRAVERSAL, false>, grid, block, s, q, ws, a);
        }
    }
    if (a.dbg_stats) {
        launch(MPV_KERNEL_DEBUG_STATS, debug_stats_kernel<E>, dim3(static_cast<unsigned>(p->B) * p->N), dim3(kTaskBlock), s, tree, a);
    }
    return hip_ok(hipGetLastError()) ? MPV_OK : MPV_ERR_HIP;
}

// ------------------------------------------------------------------ static scratch

// Scratch of mpv_verify_static: the workspace of one call, held by every device the library
// runs on until the process ends.  In host code the array's name is only a handle; its device
// address is looked up once per device (scratch_address) and only that pointer is ever used.
static __device__ __align__(256) unsigned char scratch[MPV_STATIC_WORKSPACE_BYTES];

constexpr int kMaxDevices = 64;
static std::atomic<void*> g_scratch_ptr[kMaxDevices];

// Device address of `scratch` on the current device (null + error code on failure).
static int scratch_address(void** out) {
    int dev = 0;
    if (!hip_ok(hipGetDevice(&dev))) return MPV_ERR_HIP;
    if (dev < 0 || dev >= kMaxDevices) return MPV_ERR_UNSUPPORTED;
    void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        if (!hip_ok(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch))) || !p) return MPV_ERR_HIP;
        g_scratch_ptr[dev].store(p, std::memory_order_release);     // every thread finds the same address
    }
    *out = p;
    return MPV_OK;
}

}  // namespace mpv

// ------------------------------------------------------------------ C ABI

extern "C" {

int mpv_version(void) { return MPV_ABI_VERSION; }

const char* mpv_strerror(int code) {
    switch (code) {
        case MPV_OK: return "success";
        case MPV_ERR_NULL: return "a required pointer is NULL";
        case MPV_ERR_BAD_SHAPE: return "invalid B, N, V or max_depth smaller than the tree depth";
        case MPV_ERR_BAD_TREE: return "invalid parent array (need parent[0] = -1 and 0 <= parent[n] < n)";
        case MPV_ERR_BAD_TEMPERATURE: return "temperature must be a finite number > 0";
        case MPV_ERR_BAD_METHOD: return "unknown method id";
        case MPV_ERR_BAD_DTYPE: return "unknown logit dtype";
        case MPV_ERR_WORKSPACE: return "workspace is NULL, not 256-byte aligned or too small";
        case MPV_ERR_UNSUPPORTED: return "problem exceeds MPV_MAX_NODES / MPV_MAX_CHILDREN / MPV_MAX_VOCAB, or a debug output this method does not provide was requested";
        case MPV_ERR_HIP: return "a HIP call failed (see mpv_last_hip_error)";
        case MPV_ERR_ALIGNMENT: return "logit base pointers must be 16-byte aligned";
        case MPV_ERR_BAD_TOP_P: return "top_p must lie in (0, 1]";
        default: return "unknown error code";
    }
}

int mpv_last_hip_error(void) { return mpv::g_last_hip_error; }

int mpv_workspace_bytes(const mpv_problem* problem, size_t* out) {
    if (!out) return MPV_ERR_NULL;
    mpv::Plan plan;
    const int rc = mpv::validate(problem, &plan);
    if (rc != MPV_OK) return rc;
    *out = mpv::carve(problem, nullptr, nullptr);
    return MPV_OK;
}

static int verify_with_workspace(const mpv_problem* problem, const mpv_buffers* buf, void* workspace,
                                 size_t workspace_bytes, void* hip_stream);

int mpv_verify(const mpv_problem* problem, const mpv_buffers* buf, void* workspace,
               size_t workspace_bytes, void* hip_stream) {
    return verify_with_workspace(problem, buf, workspace, workspace_bytes, hip_stream);
}

int mpv_verify_static(const mpv_problem* problem, const mpv_buffers* buf, void* hip_stream) {
    mpv::Plan plan;
    const int rc = mpv::validate(problem, &plan);
    if (rc != MPV_OK) return rc;
    if (mpv::carve(problem, nullptr, nullptr) > MPV_STATIC_WORKSPACE_BYTES) return MPV_ERR_WORKSPACE;
    void* ws = nullptr;
    const int rs = mpv::scratch_address(&ws);
    if (rs != MPV_OK) return rs;
    return verify_with_workspace(problem, buf, ws, MPV_STATIC_WORKSPACE_BYTES, hip_stream);
}

static int verify_with_workspace(const mpv_problem* problem, const mpv_buffers* buf, void* workspace,
                                 size_t workspace_bytes, void* hip_stream) {
    mpv::Plan plan;
    const int rc = mpv::validate(problem, &plan);
    if (rc != MPV_OK) return rc;
    if (!buf) return MPV_ERR_NULL;
    if (problem->B == 0) return MPV_OK;
    if (!buf->target_logits || !buf->draft_logits || !buf->tokens || !buf->uniforms || !buf->accept_len ||
        !buf->path_nodes || !buf->path_tokens || !buf->bonus_token || !buf->counters)
        return MPV_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(buf->target_logits) & 15u) || (reinterpret_cast<uintptr_t>(buf->draft_logits) & 15u))
        return MPV_ERR_ALIGNMENT;
    const size_t need = mpv::carve(problem, nullptr, nullptr);
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) || workspace_bytes < need) return MPV_ERR_WORKSPACE;

    mpv::Workspace ws;
    mpv::carve(problem, workspace, &ws);
    mpv::Args a;
    const int walk = problem->method == MPV_METHOD_NSS ? 1 : problem->method == MPV_METHOD_NAIVE ? 2
                   : problem->method == MPV_METHOD_SPECTR ? 3 : 0;
    if (walk && !buf->draw_uniforms) return MPV_ERR_NULL;
    if (walk && (buf->stats || buf->edge_probs)) return MPV_ERR_UNSUPPORTED;
    a.zt = buf->target_logits; a.zd = buf->draft_logits; a.tokens = buf->tokens; a.uniforms = buf->uniforms;
    a.draw_uniforms = buf->draw_uniforms; a.walk = walk;
    a.accept_len = buf->accept_len; a.path_nodes = buf->path_nodes; a.path_tokens = buf->path_tokens;
    a.bonus = buf->bonus_token; a.counters = buf->counters;
    a.dbg_stats = buf->stats; a.dbg_edge = buf->edge_probs; a.dbg_accept = buf->accept_prob; a.dbg_resid = buf->final_residual;
    a.B = problem->B; a.N = problem->N; a.V = problem->V; a.max_depth = problem->max_depth;
    a.k32 = static_cast<float>(1.4426950408889634 / static_cast<double>(problem->temperature));
    a.lazy = (walk || (buf->edge_probs == nullptr && buf->accept_prob == nullptr && buf->stats == nullptr)) ? 1 : 0;
    a.estimate = 0; a.reach_prob = nullptr; a.expected = nullptr;
    a.stagger_ticks = mpv::stagger_ticks(problem);
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (problem->logit_dtype == MPV_DTYPE_F32) return mpv::launch_all<mpv::ElemF32>(problem, plan, ws, a, s);
    return mpv::launch_all<mpv::ElemBF16>(problem, plan, ws, a, s);
}

int mpv_block_efficiency(const mpv_problem* problem, const void* target_logits, const void* draft_logits,
                         const int32_t* tokens, void* workspace, size_t workspace_bytes,
                         float* reach_prob, float* expected, uint32_t* counters, void* hip_stream) {
    mpv::Plan plan;
    const int rc = mpv::validate(problem, &plan);
    if (rc != MPV_OK) return rc;
    if (problem->B == 0) return MPV_OK;
    if (!target_logits || !draft_logits || !tokens || !expected || !counters) return MPV_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(target_logits) & 15u) || (reinterpret_cast<uintptr_t>(draft_logits) & 15u))
        return MPV_ERR_ALIGNMENT;
    const size_t need = mpv::carve(problem, nullptr, nullptr);
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) || workspace_bytes < need) return MPV_ERR_WORKSPACE;

    mpv::Workspace ws;
    mpv::carve(problem, workspace, &ws);
    mpv::Args a;
    a.zt = target_logits; a.zd = draft_logits; a.tokens = tokens;
    a.walk = problem->method == MPV_METHOD_NSS ? 1 : problem->method == MPV_METHOD_NAIVE ? 2
           : problem->method == MPV_METHOD_SPECTR ? 3 : 0;
    a.counters = counters;
    a.B = problem->B; a.N = problem->N; a.V = problem->V; a.max_depth = problem->max_depth;
    a.k32 = static_cast<float>(1.4426950408889634 / static_cast<double>(problem->temperature));
    a.lazy = 0;
    a.estimate = 1; a.reach_prob = reach_prob; a.expected = expected;
    a.stagger_ticks = mpv::stagger_ticks(problem);
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (problem->logit_dtype == MPV_DTYPE_F32) return mpv::launch_all<mpv::ElemF32>(problem, plan, ws, a, s);
    return mpv::launch_all<mpv::ElemBF16>(problem, plan, ws, a, s);
}


int mpv_acceptance_rates(const mpv_problem* problem, const void* target_logits, const void* draft_logits,
                         void* workspace, size_t workspace_bytes, float* alpha, uint32_t* counters, void* hip_stream) {
    mpv::Plan plan;
    const int rc = mpv::validate(problem, &plan);
    if (rc != MPV_OK) return rc;
    if (problem->method == MPV_METHOD_TRAVERSAL) return MPV_ERR_UNSUPPORTED;     // not an OTLP solver: App. C has no rate for it
    if (problem->B == 0) return MPV_OK;
    if (!target_logits || !draft_logits || !alpha || !counters) return MPV_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(target_logits) & 15u) || (reinterpret_cast<uintptr_t>(draft_logits) & 15u))
        return MPV_ERR_ALIGNMENT;
    const size_t need = mpv::carve(problem, nullptr, nullptr);
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) || workspace_bytes < need) return MPV_ERR_WORKSPACE;

    mpv::Workspace ws;
    mpv::carve(problem, workspace, &ws);
    mpv::Args a;
    a.zt = target_logits; a.zd = draft_logits;
    a.walk = problem->method == MPV_METHOD_NSS ? 1 : problem->method == MPV_METHOD_NAIVE ? 2
           : problem->method == MPV_METHOD_SPECTR ? 3 : 0;
    a.counters = counters;
    a.B = problem->B; a.N = problem->N; a.V = problem->V; a.max_depth = problem->max_depth;
    a.k32 = static_cast<float>(1.4426950408889634 / static_cast<double>(problem->temperature));
    a.lazy = 0;
    a.estimate = 2; a.alpha = alpha;
    a.stagger_ticks = mpv::stagger_ticks(problem);
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (problem->logit_dtype == MPV_DTYPE_F32) return mpv::launch_all<mpv::ElemF32>(problem, plan, ws, a, s);
    return mpv::launch_all<mpv::ElemBF16>(problem, plan, ws, a, s);
}

int mpv_timing_enable(int32_t max_launches) {
    mpv::LaunchTimer& t = mpv::g_timer;
    for (int i = 0; i < t.capacity; ++i) {
        (void)hipEventDestroy(t.start[i]);
        (void)hipEventDestroy(t.stop[i]);
    }
    delete[] t.start; delete[] t.stop; delete[] t.kernel;
    t = mpv::LaunchTimer();
    if (max_launches <= 0) return MPV_OK;
    t.start = new hipEvent_t[max_launches];
    t.stop = new hipEvent_t[max_launches];
    t.kernel = new int32_t[max_launches];
    for (int i = 0; i < max_launches; ++i) {
        if (!mpv::hip_ok(hipEventCreate(&t.start[i])) || !mpv::hip_ok(hipEventCreate(&t.stop[i]))) {
            t.capacity = i;
            mpv_timing_enable(0);
            return MPV_ERR_HIP;
        }
        t.capacity = i + 1;
    }
    t.enabled = true;
    return MPV_OK;
}

int mpv_timing_read(float* ms_out, int32_t* kernel_out, int32_t capacity, int32_t* count) {
    if (!count) return MPV_ERR_NULL;
    mpv::LaunchTimer& t = mpv::g_timer;
    const int n = t.used < capacity ? t.used : capacity;
    if (n > 0 && (!ms_out || !kernel_out)) return MPV_ERR_NULL;
    for (int i = 0; i < n; ++i) {
        float ms = 0.f;
        if (!mpv::hip_ok(hipEventElapsedTime(&ms, t.start[i], t.stop[i]))) return MPV_ERR_HIP;
        ms_out[i] = ms;
        kernel_out[i] = t.kernel[i];
    }
    *count = n;
    t.used = 0;
    return MPV_OK;
}

int mpv_row_stats(const void* logits, int32_t logit_dtype, int64_t rows, int32_t V, float temperature,
                  float* out, void* hip_stream) {
    if (!logits || !out) return MPV_ERR_NULL;
    if (rows < 0 || V < 1 || rows > 0x7fffffffLL) return MPV_ERR_BAD_SHAPE;
    if (V > MPV_MAX_VOCAB) return MPV_ERR_UNSUPPORTED;
    if (!(temperature > 0.0f) || !isfinite(temperature)) return MPV_ERR_BAD_TEMPERATURE;
    if (logit_dtype != MPV_DTYPE_F32 && logit_dtype != MPV_DTYPE_BF16) return MPV_ERR_BAD_DTYPE;
    if (rows == 0) return MPV_OK;
    const float k32 = static_cast<float>(1.4426950408889634 / static_cast<double>(temperature));
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    (void)hipGetLastError();
    if (logit_dtype == MPV_DTYPE_F32)
        hipLaunchKernelGGL((mpv::row_stats_kernel<mpv::ElemF32>), dim3(static_cast<unsigned>(rows)), dim3(mpv::kTaskBlock), 0, s,
                           static_cast<const float*>(logits), rows, V, k32, out);
    else
        hipLaunchKernelGGL((mpv::row_stats_kernel<mpv::ElemBF16>), dim3(static_cast<unsigned>(rows)), dim3(mpv::kTaskBlock), 0, s,
                           static_cast<const uint16_t*>(logits), rows, V, k32, out);
    return mpv::hip_ok(hipGetLastError()) ? MPV_OK : MPV_ERR_HIP;
}

int mpv_nucleus_mask(const void* logits, void* out, int32_t logit_dtype, int64_t rows, int32_t V,
                     float temperature, float top_p, float* threshold_out, int32_t* kept_out, void* hip_stream) {
    if (rows < 0 || V < 1) return MPV_ERR_BAD_SHAPE;
    if (V > MPV_MAX_VOCAB || rows > 0x7fffffffLL) return MPV_ERR_UNSUPPORTED;
    if (logit_dtype != MPV_DTYPE_F32 && logit_dtype != MPV_DTYPE_BF16) return MPV_ERR_BAD_DTYPE;
    if (!(temperature > 0.0f) || !isfinite(temperature)) return MPV_ERR_BAD_TEMPERATURE;
    if (!(top_p > 0.0f) || !(top_p <= 1.0f)) return MPV_ERR_BAD_TOP_P;
    if (rows == 0) return MPV_OK;
    if (!logits || !out) return MPV_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(logits) & 15u) || (reinterpret_cast<uintptr_t>(out) & 15u)) return MPV_ERR_ALIGNMENT;
    const float k32 = static_cast<float>(1.4426950408889634 / static_cast<double>(temperature));
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    (void)hipGetLastError();
    const dim3 grid(static_cast<unsigned>(rows)), block(mpv::kNucleusBlock);
    // top_p = 1 keeps every token: a threshold no mass can miss
    const float p = top_p < 1.0f ? top_p : 0.0f;
    if (logit_dtype == MPV_DTYPE_F32)
        hipLaunchKernelGGL((mpv::nucleus_kernel<mpv::ElemF32>), grid, block, 0, s, static_cast<const float*>(logits),
                           static_cast<float*>(out), rows, V, k32, p, top_p < 1.0f ? 0 : 1, threshold_out, kept_out);
    else
        hipLaunchKernelGGL((mpv::nucleus_kernel<mpv::ElemBF16>), grid, block, 0, s, static_cast<const uint16_t*>(logits),
                           static_cast<uint16_t*>(out), rows, V, k32, p, top_p < 1.0f ? 0 : 1, threshold_out, kept_out);
    return mpv::hip_ok(hipGetLastError()) ? MPV_OK : MPV_ERR_HIP;
}

int mpv_fill_uniforms(uint64_t seed, int64_t count, float* d_u, void* hip_stream) {
    if (count < 0) return MPV_ERR_BAD_SHAPE;
    if (count == 0) return MPV_OK;
    if (!d_u) return MPV_ERR_NULL;
    const int threads = 256;
    const int64_t blocks = (count + threads - 1) / threads;
    if (blocks > 0x7fffffffLL) return MPV_ERR_UNSUPPORTED;
    (void)hipGetLastError();
    hipLaunchKernelGGL(mpv::fill_uniforms_kernel, dim3(static_cast<unsigned>(blocks)), dim3(threads), 0,
                       static_cast<hipStream_t>(hip_stream), seed, count, d_u);
    return mpv::hip_ok(hipGetLastError()) ? MPV_OK : MPV_ERR_HIP;
}

}  // extern "C"
