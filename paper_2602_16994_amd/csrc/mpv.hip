// mpv.hip -- kernels and C ABI of the tree-verification library (gfx950 only).
//
// Path of one mpv_verify call (all on the caller's stream):
//   init_kernel            zero counters, default the per-node results, queue the first tasks
//   node_task_kernel       persistent workgroups of 256 lanes, three per compute unit, grouped in
//                          TEAMS of G workgroups that take tasks from a queue until none are left.
//                          A team splits every logit row by vocabulary range: each member keeps its
//                          part of the task's (target, draft) row pair on chip (registers + LDS),
//                          and every V-wide sum is a local partial plus one exchange of a few
//                          words between the members (through memory; about a microsecond).
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
//                            tree: the uniform-dependent walk, then the team draws the bonus
//                            token by inverse CDF from the residual of the stopping node.
//                            (NSS, Naive, SpecTr: one per draw of the token-following walk.)
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

// Node numbers are below MPV_MAX_NODES = 64: one byte each (the tables live in LDS, where the three
// workgroups of a compute unit have 53 KB each).
struct TreeDesc {
    int32_t N;
    int8_t parent[MPV_MAX_NODES];
    int8_t nchild[MPV_MAX_NODES];
    int8_t child_off[MPV_MAX_NODES];     // start of the node's children in child_list
    int8_t child_list[MPV_MAX_NODES];    // children of node 0, of node 1, ... ascending
    int8_t depth[MPV_MAX_NODES];
    int8_t postorder[MPV_MAX_NODES];     // depth-first, children (in list order) before their parent; root last
    int8_t rank[MPV_MAX_NODES];          // position of the node in postorder
    int8_t sub_lo[MPV_MAX_NODES];        // the node's subtree is postorder[sub_lo[n] .. rank[n]]
    int8_t cls[MPV_MAX_NODES];           // priority class of the node's task (see QueuePlan)
    int8_t pad[MPV_MAX_NODES];
    int32_t class_off[8];                // QueuePlan::off again, for the kernels that read the tables from memory
};
static_assert(MPV_MAX_NODES <= 127 && sizeof(TreeDesc) % 4 == 0, "node numbers must fit a signed byte");

constexpr int kMaxClasses = 4;
static_assert(kMaxClasses + 1 <= 8, "TreeDesc::class_off is too short");

// The task queue is one first-in-first-out queue per priority class; a free team is
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
    int32_t teams;                       // teams of the launch (the grid is teams * team_size workgroups)
    int32_t team_size;                   // G: workgroups that share one task
    int32_t part_vecs;                   // 16-byte vectors of a row per member (a multiple of 64)
    int32_t same_xcd;                    // members of a team are 8 workgroup numbers apart (one chiplet, its L2)
    // Traversal, only what is needed, no team to spare: the node where the tree branches
    // (-1: not used) first handles its first child only; the rest of its work (a second task:
    // "resumed") is started when that child's subtree, split_mask in postorder positions, turns
    // out to be rejected as a whole.
    int32_t split_node;
    unsigned long long split_mask;

};

constexpr int kMaxTeam = 16;                          // workgroups per team, at most
constexpr int kExchWords = 8;                         // 64-bit words one member hands over per exchange
constexpr int kMaxGrid = 768;                        // workgroups of a launch, at most (three per compute unit)

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
    // [2] exit: set when nothing is left, [3] lock: held by the team leader that is dispatching,
    // [4 + c] tail of class c: entries appended, [4 + kMaxClasses + c] head of class c: entries handed out,
    // [4 + 2 kMaxClasses] teams left waiting after the last round of dispatching (a hint)
    int32_t* qctl;
    int32_t* mailbox;    // [teams] kMailboxAbsent until every member has started, then kMailboxWaiting /
                         // kMailboxSoon, or the task handed to that team
    // Per tree, one bit per node at the node's position in postorder: `known` = the outcome of
    // the node's test is settled, `acc` = it is "accepted" (valid once known).  `decided` = the
    // sampling task has been queued (and, when only what the rule needs is computed, the
    // tree's remaining node tasks are cancelled).
    unsigned long long* known;
    unsigned long long* acc;
    int32_t* decided;
    int32_t* cur;        // [B] token-following walks: the node the walk has reached
    TreeDesc* tree;      // the tree tables, written by init_kernel for the kernel that follows
    // Teams.  exch: [team][2][member][kExchWords] words of (sequence number << 32 | 32 bits of payload);
    // team_task: [team][2] the task the leader has taken and its flags, same packing; arrived: members
    // of the team that have started.
    unsigned long long* exch;
    unsigned long long* team_task;
    int32_t* arrived;
    struct Launch* launch;   // what node_task_kernel is launched with, written by init_kernel
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
    // Expected block efficiency instead of a verification (Sec. 5, Eq. 1-3): every node task runs
    // (lazy = 0), no uniforms are read, and what would be a tree's sampling task turns the per-node
    // results into reach probabilities.  reach_prob [B,N] may be null; expected [B].
    // estimate = 2: acceptance rates instead (App. C): per internal node, from its two rows and its
    // number of children alone; no tokens are read, nothing follows the node tasks.  alpha [B,N].
    int32_t estimate = 0;
    int32_t keep_counters = 0;   // the call continues an earlier one: init_kernel leaves the counters as they are
    int32_t reserved = 0;
    float* reach_prob = nullptr;
    float* expected = nullptr;
    float* alpha = nullptr;
    // Trees of distinct contexts, SpecTr: [B,N], the node an accepted child entry stands for (itself unless the
    // entry repeats a token drafted earlier under the same node); null: every entry stands for itself.
    const int32_t* context_node = nullptr;
};

// Everything node_task_kernel needs to know, in one block of the workspace: the kernel and the
// functions it calls read it through one pointer (as kernel arguments, passed on by reference, the
// three structures were copied into every lane's private memory).
struct Launch {
    QueuePlan q;
    Workspace ws;
    Args a;
};

constexpr int kTaskBlock = 256;
constexpr int kTaskWaves = kTaskBlock / kWave;
constexpr int kTaskUnroll = 4;
// node tasks keep their part of a row pair on chip: per lane and row, kRegVecs 16-byte vectors in
// registers and kLdsVecs in LDS
constexpr int kRegVecs = 6;
constexpr int kLdsVecs = 6;
constexpr int kPartCapacity = (kRegVecs + kLdsVecs) * kTaskBlock;     // vectors of a row one member keeps
// upper bound on the polls of a dependency flag (about a second); see node_task_kernel
constexpr int kMaxSpins = 1 << 20;
// no wait inside a launch outlasts this (wall clock, 100 MHz ticks: 2 s)
constexpr long long kLaunchTimeoutTicks = 200000000ll;
// bit pattern (a NaN) of a starting weight that has not been published yet
constexpr unsigned long long kNotReady = ~0ull;
// wave tiles of the bonus sampler: 64 16-byte vectors; float rows have the smallest tiles
constexpr int kMaxTiles = MPV_MAX_VOCAB / (kWave * 4);
// task hand-over between the dispatcher and the teams (see "task queue")
constexpr int kMailboxWaiting = -1;                  // the team is idle
constexpr int kMailboxSoon = -2;                     // the team has asked ahead: it will be free shortly
constexpr int kMailboxAbsent = -3;                   // not every member of the team has started yet
constexpr int kTaskExit = -1;                         // what a leader's wait returns when all is done
constexpr int kWorkerSlots = 8;                       // mailboxes per dispatcher lane
constexpr int kMaxTeams = kWave * kWorkerSlots;
constexpr int kKindAcceptance = 100;                   // node_task_kernel instantiation for the acceptance rates (see there)

// LDS of node_task_kernel that the functions it calls use as well (file scope, so that they address
// it as LDS and not through generic pointers)
struct TaskShared {
    double scratch[2 * kTaskWaves];               // block reductions of the stand-alone helpers
    double part[kTaskWaves][4];                   // per-wave partial sums of a team reduction
    float partf[kTaskWaves][2];                   // per-wave reference exponents of the statistics
    unsigned words[kMaxTeam * kExchWords];        // what the members exchanged last
    int dead;
};
__shared__ TaskShared g_sh;
// the launch parameters (copied from the workspace at the start of node_task_kernel)
__shared__ __align__(16) int g_launch_words[sizeof(Launch) / sizeof(int)];
__device__ __forceinline__ const Launch& lds_launch() { return *reinterpret_cast<const Launch*>(g_launch_words); }
// the part of the row pair kept in LDS (target slots, then draft slots); the sampling task's table
// of tile masses uses the same memory
__shared__ uint4 g_rows[2 * kLdsVecs * kTaskBlock];
static_assert(sizeof(g_rows) >= kMaxTiles * sizeof(float), "tile masses do not fit in the kept-row LDS");
// the tree tables (copied from the workspace at the start of node_task_kernel)
__shared__ TreeDesc g_tree;

// A value that is the same in every lane, for the compiler to keep in scalar registers.  Needed
// wherever a function that is not inlined receives it: arguments arrive in vector registers.
__device__ __forceinline__ int uniform_i32(int x) { return __builtin_amdgcn_readfirstlane(x); }
template <class P>
__device__ __forceinline__ P* uniform_ptr(P* p) {
    const unsigned long long v = reinterpret_cast<unsigned long long>(p);
    const unsigned lo = static_cast<unsigned>(__builtin_amdgcn_readfirstlane(static_cast<int>(v)));
    const unsigned hi = static_cast<unsigned>(__builtin_amdgcn_readfirstlane(static_cast<int>(v >> 32)));
    return reinterpret_cast<P*>((static_cast<unsigned long long>(hi) << 32) | lo);
}
template <class S>
__device__ __forceinline__ S uniform_struct(const S& s) {
    static_assert(sizeof(S) % 4 == 0, "whole words only");
    S out;
    const int* src = reinterpret_cast<const int*>(&s);
    int* dst = reinterpret_cast<int*>(&out);
#pragma unroll
    for (int i = 0; i < static_cast<int>(sizeof(S) / 4); ++i) dst[i] = __builtin_amdgcn_readfirstlane(src[i]);
    return out;
}

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
    {   // the launch block of the next kernel
        struct Words { Launch l; };
        const int groups = gridDim.x * gridDim.y;
        int* dst = reinterpret_cast<int*>(ws.launch);
        const int me = blockIdx.y * gridDim.x + blockIdx.x;
        const int nq = static_cast<int>(sizeof(QueuePlan) / sizeof(int)), nw = static_cast<int>(sizeof(Workspace) / sizeof(int));
        const int na = static_cast<int>(sizeof(Args) / sizeof(int));
        static_assert(sizeof(QueuePlan) % 8 == 0 && sizeof(Workspace) % 8 == 0 && sizeof(Args) % 8 == 0, "Launch has no padding between its members");
        for (int w = me; w < nq + nw + na; w += groups) {
            int v;
            if (w < nq) v = reinterpret_cast<const int*>(&q)[w];
            else if (w < nq + nw) v = reinterpret_cast<const int*>(&ws)[w - nq];
            else v = reinterpret_cast<const int*>(&a)[w - nq - nw];
            if (threadIdx.x == 0) dst[w] = v;
        }
    }
    {   // team words: every sequence number starts at 0, nobody has arrived
        const int stride = gridDim.x * gridDim.y * blockDim.x;
        const int me = (blockIdx.y * gridDim.x + blockIdx.x) * blockDim.x + threadIdx.x;
        for (int w = me; w < kMaxGrid * 2 * kExchWords; w += stride) ws.exch[w] = 0ull;
        for (int w = me; w < kMaxTeams * 2; w += stride) ws.team_task[w] = 0ull;
        for (int w = me; w < kMaxTeams; w += stride) { ws.arrived[w] = 0; ws.mailbox[w] = kMailboxAbsent; }
    }
    if (n == 0) {
        if (i < MPV_COUNTER_COUNT && !a.keep_counters) a.counters[i] = 0u;
        if (i == 0) { ws.qctl[0] = q.init_total; ws.qctl[1] = 0; ws.qctl[2] = 0; ws.qctl[3] = 0; ws.qctl[4 + 2 * kMaxClasses] = 0; }
        for (int c = 0; c < kMaxClasses; ++c)
            if (i == 0) {
                ws.qctl[4 + c] = (c < q.nclass) ? q.init_tail[c] : 0;
                ws.qctl[4 + kMaxClasses + c] = 0;
            }
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
            if (q.root_is_leaf) ws.queue[q.off[0] + i] = a.B * a.N + i;
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
    }
}

// ------------------------------------------------------------------ task queue
//
// node_task_kernel is launched with three workgroups per compute unit at most, grouped in teams;
// each team runs tasks until told to exit.  A team takes part only once every member has
// started (the last to arrive opens the team's mailbox), so a task is only ever handed to
// workgroups that are running, whatever else occupies the device.  A task is appended only when
// everything it needs has been published, so every queued task can run at once, on any team.
//   append:   appended++, then slot = tail++ of the class, then the entry is written.
//   request:  mailbox[team] = "soon" when a team asks ahead, before the last sweep of its
//             current task (the answer is then usually there when it is done), "waiting" once
//             it has nothing to do.  Idle teams are served before those that asked ahead.
//   dispatch: a leader that has nothing to do takes the dispatcher lock if it is free and,
//             with its first wave, hands queued tasks to waiting teams (its own included)
//             in priority order (class, then age), until it has a task of its own; then it
//             releases the lock.  Those that find the lock taken poll their mailbox.  If every
//             team is busy nobody dispatches, and nobody needs to.  Node tasks of trees
//             whose outcome is settled are dropped here when only what is needed is computed.
//   end:      nothing queued and completed == appended, with appended read before and after
//             completed and unchanged: no task is queued, handed out or running, so nothing
//             can be appended any more; the dispatching leader sets the exit flag.  A
//             task's appends are performed before its completed++.
// A team may also run a task it has produced itself straight away (counted in appended,
// never queued).  Every wait is bounded.  Only the leader (member 0) of a team talks to the queue.

__device__ __forceinline__ int ld_relaxed(const int32_t* p) {
    return __hip_atomic_load(as_global(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long ld_relaxed(const unsigned long long* p) {
    return __hip_atomic_load(as_global(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_relaxed(int32_t* p, int v) {
    __hip_atomic_store(as_global(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_relaxed(unsigned long long* p, unsigned long long v) {
    __hip_atomic_store(as_global(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// The read-modify-write operations of the task kernels (relaxed, device scope, like HIP's own of
// these names, which they hide inside this namespace) on pointers known to be global.
__device__ __forceinline__ int atomicAdd(int* p, int v) {
    return __hip_atomic_fetch_add(as_global(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned atomicAdd(unsigned* p, unsigned v) {
    return __hip_atomic_fetch_add(as_global(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long atomicOr(unsigned long long* p, unsigned long long v) {
    return __hip_atomic_fetch_or(as_global(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ int atomicCAS(int* p, int expected, int desired) {
    __hip_atomic_compare_exchange_strong(as_global(p), &expected, desired, __ATOMIC_RELAXED, __ATOMIC_RELAXED,
                                         __HIP_MEMORY_SCOPE_AGENT);
    return expected;
}
// all loads, stores and atomics issued so far by this lane have been performed
__device__ __forceinline__ void wait_memory() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// Append one task to class c (one lane).  What the task needs and this lane has stored before
// is performed before the task can be handed out (the wait below covers it).
__device__ __forceinline__ void append_task(const TreeDesc& tree, const Workspace& ws, int c, int entry) {
    (void)atomicAdd(&ws.qctl[0], 1);
    wait_memory();                                    // counted before it can be handed out (and finished)
    const int slot = atomicAdd(&ws.qctl[4 + c], 1);
    const int first = tree.class_off[c], end = tree.class_off[c + 1];
    if (slot < end - first) st_relaxed(&ws.queue[first + slot], entry);
}

// One round of dispatching, by a whole wave that holds the lock.  Lane c keeps the head of
// class c in `head`; lane l looks after the teams l, l + 64, ...  Returns true when
// everything is finished (the exit flag has been set).
__device__ __forceinline__ bool dispatch_round(const QueuePlan& q, const TreeDesc& tree, const Workspace& ws, const Args& a, bool drop_settled,
                               int& head, long long t_begin) {
    __shared__ int sh_head[kMaxClasses], sh_before[kMaxClasses + 1];
    const int lane = threadIdx.x;
    const int workers = q.teams;
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
            if (!done && wall_clock64() - t_begin > kLaunchTimeoutTicks) {
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
    // Requester number r gets queued task number r (in class, age order); the idle teams
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

// The next task of this team, or kTaskExit; called by every lane of the leader's first wave, returns
// the same value in each.  The team has asked (its mailbox says "waiting" or already holds
// the answer).  `previous` is the task it took from the mailbox last: until the request has
// reached memory the mailbox may still show it (no entry is ever handed out twice, so the
// value is unambiguous).
__device__ __attribute__((noinline)) int acquire_task(int team_in, int previous_in, bool drop_settled_in, long long t_start) {
    const Args& a = lds_launch().a;
    const Workspace& ws = lds_launch().ws;
    const QueuePlan& q = lds_launch().q;
    const TreeDesc& tree = g_tree;
    const int team = uniform_i32(team_in), previous = uniform_i32(previous_in);
    const bool drop_settled = uniform_i32(drop_settled_in ? 1 : 0) != 0;
    const int lane = threadIdx.x;
    int32_t* const box = &ws.mailbox[team];
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
        // (a team whose mailbox is still "absent" cannot be handed anything: it does not dispatch either)
        if (lane == 0 && lk == 0 && t != kMailboxAbsent) got = (atomicCAS(&ws.qctl[3], 0, 1) == 0) ? 1 : 0;
        if (__builtin_amdgcn_readfirstlane(got)) {
            // the previous holder wrote the heads before it released the lock
            int head = (lane < q.nclass) ? ld_relaxed(&ws.qctl[4 + kMaxClasses + lane]) : 0;
            int result = kTaskExit;
            for (;;) {
                const bool finished = dispatch_round(q, tree, ws, a, drop_settled, head, t_start);
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
        if (wall_clock64() - t_start > kLaunchTimeoutTicks) break;
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
    __hip_atomic_store(as_global(reinterpret_cast<unsigned long long*>(p)),
                       static_cast<unsigned long long>(__double_as_longlong(v)), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ double ld_shared_f64(const double* p) {
    return __longlong_as_double(static_cast<long long>(__hip_atomic_load(
        as_global(reinterpret_cast<const unsigned long long*>(p)), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)));
}

// ------------------------------------------------------------------ teams
//
// The G members of a team run the same task in lockstep on different vocabulary ranges: they
// execute the same scalar code on the same numbers (exchanged sums are added in member order
// by every member, so they are bitwise equal everywhere) and therefore take the same branches;
// side effects (results, queue, counters) are the leader's (member 0).  What the leader alone
// can know (the task, whether teams are idle, a starting weight) travels with the task word or
// with the first exchange of the task.
// An exchange: every member writes up to kExchWords words into its own 64-byte line of the
// team's area, each word tagged with the number of the exchange, and polls the other lines until
// every word carries that number.  Two areas alternate: a member can be at most one exchange
// ahead of the slowest (it needs everybody's words of exchange s to finish s), so the words
// of exchange s are never overwritten before everybody has read them.

struct Team {
    int id, member, size;
    unsigned seq;                    // exchanges done
    unsigned tseq;                   // task words seen
    unsigned long long* area;        // [2][size][kExchWords]
    unsigned long long* task_word;   // [2]
    long long t_start;               // wall clock at the start of the launch
    int dead;                        // a partner never answered: results are invalid, every wait is skipped
};

// What a workgroup carries from task to task, kept in LDS: the functions that run the tasks are
// not inlined, and state handed to them by reference would live in each lane's private memory.
// Written by the first lane of the first wave only (between two barriers of the task loop);
// whoever needs it takes a copy into registers.
struct LoopState {
    Team team;
    int asked;            // the leader has asked for its next task (mailbox says waiting or soon)
    int own_task;         // leader: a task the team produced for itself, already announced (-1: none);
                          // member: the task it has already heard of (kNothingHeard: none)
    int own_flags;
    int previous_task;    // last task taken from the mailbox
};
__shared__ LoopState g_loop;
constexpr int kNothingHeard = -4;

// First wave only.  Lane w < kExchWords brings `mine`, its 32 bits of payload.  On return
// g_sh.words[m * kExchWords + w] holds member m's word w (visible to the other waves after the
// caller's next barrier) and g_sh.dead says whether a partner failed to answer.
__device__ __forceinline__ void exchange_words(const Team& t, unsigned mine) {
    const Workspace& ws = lds_launch().ws;
    const Args& a = lds_launch().a;
    const int lane = threadIdx.x;
    if (t.size == 1) {
        if (lane < kExchWords) g_sh.words[lane] = mine;
        if (lane == 0) g_sh.dead = t.dead;
        return;
    }
    unsigned long long* base = t.area + static_cast<size_t>(t.seq & 1u) * t.size * kExchWords;
    const unsigned long long tag = static_cast<unsigned long long>(t.seq) << 32;
    if (lane < kExchWords) st_relaxed(base + t.member * kExchWords + lane, tag | mine);
    int dead = t.dead;
    for (int w = lane; w < t.size * kExchWords; w += kWave) {
        unsigned long long v = 0ull;
        while (!dead) {
            v = ld_relaxed(base + w);
            if ((v >> 32) == (tag >> 32)) break;
            if (wall_clock64() - t.t_start > kLaunchTimeoutTicks) { dead = 1; break; }
            __builtin_amdgcn_s_sleep(1);
        }
        g_sh.words[w] = dead ? 0u : static_cast<unsigned>(v);
    }
    const int any_dead = __ballot(dead != 0) != 0ull;
    if (lane == 0) {
        g_sh.dead = any_dead;
        if (any_dead && !t.dead) {
            atomicAdd(&a.counters[MPV_COUNTER_DEPENDENCY_TIMEOUT], 1u);
            st_relaxed(&ws.qctl[2], 1);                // everybody leaves at the next occasion
        }
    }
}

// All lanes of the workgroup: one exchange of raw words (lane w < kExchWords of the first wave
// brings `mine`); afterwards every lane may read g_sh.words.
__device__ __forceinline__ void team_exchange(Team& t, unsigned mine) {
    t.seq++;
    __syncthreads();                                  // earlier readers of g_sh.words are done
    if (threadIdx.x < kWave) exchange_words(t, mine);
    __syncthreads();
    t.dead = g_sh.dead;
}

__device__ __forceinline__ unsigned half_of(double v, int hi) {
    return static_cast<unsigned>(hi ? __double2hiint(v) : __double2loint(v));
}
__device__ __forceinline__ double double_at(const unsigned* words, int member, int pair) {
    return __hiloint2double(static_cast<int>(words[member * kExchWords + 2 * pair + 1]),
                            static_cast<int>(words[member * kExchWords + 2 * pair]));
}

// Sums of up to four per-lane values over every lane of every member of the team: wave sums, the
// four waves and then the members added in a fixed order, so every lane of every member gets the
// same bits.  Two barriers: wave partials -> (first wave: block total, exchange) -> everybody reads.
template <int COUNT>
__device__ __forceinline__ void team_sum(Team& t, double (&v)[COUNT]) {
    static_assert(COUNT * 2 <= kExchWords && COUNT <= 4, "too many values for one exchange");
    const int wave = threadIdx.x / kWave, lane = threadIdx.x & (kWave - 1);
    t.seq++;
#pragma unroll
    for (int i = 0; i < COUNT; ++i) {
        const double w = wave_sum(v[i]);
        if (lane == 0) g_sh.part[wave][i] = w;
    }
    __syncthreads();
    if (wave == 0) {
        unsigned mine = 0u;
        if (lane < 2 * COUNT) {
            const int i = lane >> 1;
            double b = g_sh.part[0][i];
#pragma unroll
            for (int w = 1; w < kTaskWaves; ++w) b += g_sh.part[w][i];
            mine = half_of(b, lane & 1);
        }
        exchange_words(t, mine);
    }
    __syncthreads();
    t.dead = g_sh.dead;
#pragma unroll
    for (int i = 0; i < COUNT; ++i) {
        double s = 0.0;
        for (int m = 0; m < t.size; ++m) s += double_at(g_sh.words, m, i);
        v[i] = uniform_f64(s);
    }
}

// The leader tells the others which task it has taken.  Every task announced this way contains at
// least one exchange, so the leader cannot announce the next before everybody has read this one.
__device__ __forceinline__ void team_announce(Team& t, int task, int flags) {
    t.tseq++;
    if (t.size == 1) return;
    if (threadIdx.x < 2) {
        const unsigned long long tag = static_cast<unsigned long long>(t.tseq) << 32;
        st_relaxed(t.task_word + threadIdx.x, tag | static_cast<unsigned>(threadIdx.x == 0 ? task : flags));
    }
}
// The others wait for it (first wave; returns the same in every lane).  kTaskExit on a timeout.
__device__ __forceinline__ int team_listen(Team& t, int& flags, const Workspace& ws) {
    t.tseq++;
    unsigned long long v = 0ull;
    int ok = 1;
    if (threadIdx.x < 2) {
        for (;;) {
            v = ld_relaxed(t.task_word + threadIdx.x);
            if ((v >> 32) == t.tseq) break;
            if (wall_clock64() - t.t_start > kLaunchTimeoutTicks) { ok = 0; break; }
            __builtin_amdgcn_s_sleep(2);
        }
    }
    const int all_ok = __ballot(!ok) == 0ull;
    const int task = __builtin_amdgcn_readlane(static_cast<int>(static_cast<unsigned>(v)), 0);
    flags = __builtin_amdgcn_readlane(static_cast<int>(static_cast<unsigned>(v)), 1);
    return all_ok ? task : kTaskExit;
}

// ------------------------------------------------------------------ node task

// Double-precision scalar steps between the sweeps, as calls: their registers are then theirs alone
// and the part of the row pair a task keeps in registers stays where it is.
__device__ __forceinline__ double cold_exp2(double x) { return exp2(x); }
// 2^x for a probability (x <= a few): the whole part of x goes into the exponent, the rest through
// the hardware's float 2^f (relative error about 1e-7, far inside what a test probability needs):
// a dozen instructions on the first wave's path instead of the library routine's hundred.
__device__ __forceinline__ double probability_exp2(double x) {
    if (!(x > -1000.0)) return 0.0;                    // (also -inf and NaN)
    const double n = rint(x);
    const float f = static_cast<float>(x - n);         // [-0.5, 0.5]
    return ldexp(static_cast<double>(fast_exp2(f)), static_cast<int>(n));
}
__device__ __forceinline__ double cold_log2(double x) { return log2(x); }
__device__ __forceinline__ ResidualConsts cold_residual_consts(double At, double Ad, double c) { return residual_consts(At, Ad, c); }
// x^k for a small whole k
__device__ __forceinline__ double int_power(double x, int k) {
    double r = 1.0;
    for (int i = 0; i < k; ++i) r *= x;
    return r;
}

// task word flags (leader -> members)
constexpr int kFlagIdle = 1;          // teams were idle after the last round of dispatching

// (defined below) walk and bonus token of tree b, or one draw of a token-following walk, by the
// whole team; returns the task that follows from it (-1: none; the same in every lane of every member)
template <class E, int METHOD>
__device__ __attribute__((noinline)) int sample_task(int b_in);

// (defined below) expected block efficiency of tree b from the per-node results, by the first wave
template <int METHOD>
__device__ __forceinline__ void estimate_wave(const TreeDesc& tree, const Workspace& ws, const Args& a, int b);

// Softmax statistics of the task's two rows from the lanes' states (sum_v 2^(z_v k32 - mk) against
// each lane's own reference mk): lanes are brought to their wave's largest reference, waves to the
// workgroup's, members to the team's; one exchange, which also carries the node's starting weight
// from the leader (*a0_lds, LDS, written before the call; what the other members pass is ignored).
// Every lane of every member gets the same bits.
__device__ __forceinline__ void team_stats(Team& t, const OnlineLse& lt, const OnlineLse& ld, const double* a0_lds,
                                           double& At, double& Ad, double& a0) {
    const int wave = threadIdx.x / kWave, lane = threadIdx.x & (kWave - 1);
    t.seq++;
    const float Mt_w = wave_max(lt.mk), Md_w = wave_max(ld.mk);
    const double st_w = wave_sum((lt.s > 0.f) ? static_cast<double>(lt.s * fast_exp2(lt.mk - Mt_w)) : 0.0);
    const double sd_w = wave_sum((ld.s > 0.f) ? static_cast<double>(ld.s * fast_exp2(ld.mk - Md_w)) : 0.0);
    if (lane == 0) {
        g_sh.partf[wave][0] = Mt_w; g_sh.partf[wave][1] = Md_w;
        g_sh.part[wave][0] = st_w; g_sh.part[wave][1] = sd_w;
    }
    __syncthreads();
    if (wave == 0) {
        float Mt = g_sh.partf[0][0], Md = g_sh.partf[0][1];
#pragma unroll
        for (int w = 1; w < kTaskWaves; ++w) { Mt = fmaxf(Mt, g_sh.partf[w][0]); Md = fmaxf(Md, g_sh.partf[w][1]); }
        double st = 0.0, sd = 0.0;
#pragma unroll
        for (int w = 0; w < kTaskWaves; ++w) {
            st += g_sh.part[w][0] * static_cast<double>(fast_exp2(g_sh.partf[w][0] - Mt));
            sd += g_sh.part[w][1] * static_cast<double>(fast_exp2(g_sh.partf[w][1] - Md));
        }
        const double a0_mine = *a0_lds;
        unsigned mine = 0u;
        switch (lane) {
            case 0: mine = __float_as_uint(Mt); break;
            case 1: mine = __float_as_uint(Md); break;
            case 2: mine = half_of(st, 0); break;
            case 3: mine = half_of(st, 1); break;
            case 4: mine = half_of(sd, 0); break;
            case 5: mine = half_of(sd, 1); break;
            case 6: mine = half_of(a0_mine, 0); break;
            case 7: mine = half_of(a0_mine, 1); break;
            default: break;
        }
        exchange_words(t, mine);
    }
    __syncthreads();
    t.dead = g_sh.dead;
    float MT = OnlineLse::kFloor, MD = OnlineLse::kFloor;
    for (int m = 0; m < t.size; ++m) {
        MT = fmaxf(MT, __uint_as_float(g_sh.words[m * kExchWords]));
        MD = fmaxf(MD, __uint_as_float(g_sh.words[m * kExchWords + 1]));
    }
    double ST = 0.0, SD = 0.0;
    for (int m = 0; m < t.size; ++m) {
        ST += double_at(g_sh.words, m, 1) * static_cast<double>(fast_exp2(__uint_as_float(g_sh.words[m * kExchWords]) - MT));
        SD += double_at(g_sh.words, m, 2) * static_cast<double>(fast_exp2(__uint_as_float(g_sh.words[m * kExchWords + 1]) - MD));
    }
    At = uniform_f64(static_cast<double>(MT) + cold_log2(ST));
    Ad = uniform_f64(static_cast<double>(MD) + cold_log2(SD));
    a0 = uniform_f64(double_at(g_sh.words, 0, 3));
}

// One node task (or the resumed task of the node where the tree branches), by every member of the
// team.  A function of its own, not inlined: what it keeps in registers (its part of the row pair)
// then competes only with its own scalar steps for registers, not with the dispatcher or the sampler.
//
// Inside a workgroup the four waves split the work in another way as well: all four sweep their
// share of the part, but everything scalar (statistics, weights, the child loop, the exchange with
// the other members, what follows from the task) is the first wave's alone.  The other waves wait
// at a barrier for the next sweep's constants: they issue no instruction meanwhile, which leaves
// the compute unit to the sweeps of the other workgroups that live on it.
//   first wave:   ... scalar step ... | write command | barrier B | sweep | partial | barrier A | read partials ...
//   other waves:                                      | barrier B | sweep | partial | barrier A | (loop)
// asked / own_task / own_flags: the leader's notes for the task loop (has the team asked for its
// next task; the task it is to run next, already announced to the team, and its flags); only the
// first wave's copies matter.

// The barrier between the waves of a workgroup inside a node task.  What the waves hand each other
// there goes through LDS only (the command, partial sums, the children's scalars), so the barrier
// waits for this wave's LDS operations and nothing else: __syncthreads() would also wait for every
// global load in flight, i.e. for the rows of the next task that have just been asked for.
__device__ __forceinline__ void task_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

constexpr int kCmdTask = 5;
constexpr int kCmdDone = 0;          // the task is over
constexpr int kCmdMass = 1;          // sum (p - rho q)_+
constexpr int kCmdMassSlope = 2;     // the same and sum_{p > rho q} rho q       (SpecTr's root search)
constexpr int kCmdAcceptance = 3;    // the NSS / Naive acceptance-rate sum      (acceptance rates only)

struct SweepCmd {
    int kind;
    float nAt, nAd, rho;             // constants of the residual sweeps
    float sp, sq;                    // acceptance sweep: scale factors of p and q
    int m, naive;                    // acceptance sweep: exponent, which formula (kCmdTask: m = the task)
    int next;                        // a sweep: the task this team goes on with when the sweep was the
                                     // current task's last (-1: not known); each wave asks for its share
                                     // of that task's rows as soon as it is done with its share of the sweep
};
__shared__ SweepCmd g_cmd;

// One sweep over the part on chip as the command says; the wave's partial sums go to g_sh.part.
template <class E, int KIND, class PAIR>
__device__ __forceinline__ void run_sweep(PAIR& pair, const SweepCmd& cmd, float k32, int wave, int lane) {
    constexpr bool ACCEPT = KIND == kKindAcceptance;
    constexpr bool SLOPE = KIND != MPV_METHOD_TRAVERSAL;      // SpecTr's search exists in the top-down kernels only
    double s0 = 0.0, s1 = 0.0;
    if (SLOPE && cmd.kind == kCmdMassSlope) {
        ResidualMassSlopeRawF<E> f;
        f.init();
        f.k32 = k32; f.nAt = cmd.nAt; f.nAd = cmd.nAd; f.rho = cmd.rho;
        pair.replay(f);
        s0 = static_cast<double>(f.acc0) + static_cast<double>(f.acc1);
        s1 = static_cast<double>(f.q0) + static_cast<double>(f.q1);
    } else if (ACCEPT && cmd.kind == kCmdAcceptance) {
        AcceptanceF<E> f;
        f.init(k32, cmd.nAt, cmd.nAd, cmd.sp, cmd.sq, cmd.m, cmd.naive != 0);
        pair.replay(f);
        s0 = static_cast<double>(f.acc0) + static_cast<double>(f.acc1);
    } else {
        ResidualMassRawF<E> f;
        f.init(k32, cmd.nAt, cmd.nAd, cmd.rho);
        pair.replay(f);
        s0 = f.total();
    }
    s0 = wave_sum(s0);
    if (SLOPE) s1 = wave_sum(s1);
    if (lane == 0) { g_sh.part[wave][0] = s0; g_sh.part[wave][1] = s1; }
}

// First wave, after barrier A: the workgroup's sums of the last sweep, exchanged and added over the
// team in member order.  Every lane of the first wave of every member gets the same bits.
__device__ __forceinline__ void collect_sums(Team& t, double& s0, double& s1) {
    const int lane = threadIdx.x;
    t.seq++;
    unsigned mine = 0u;
    if (lane < 4) {
        const int i = lane >> 1;
        double b = g_sh.part[0][i];
#pragma unroll
        for (int w = 1; w < kTaskWaves; ++w) b += g_sh.part[w][i];
        mine = half_of(b, lane & 1);
    }
    exchange_words(t, mine);
    __builtin_amdgcn_wave_barrier();
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");       // the wave's own LDS writes, before its reads
    t.dead = g_sh.dead;
    double a = 0.0, b = 0.0;
    for (int m = 0; m < t.size; ++m) { a += double_at(g_sh.words, m, 0); b += double_at(g_sh.words, m, 1); }
    s0 = uniform_f64(a);
    s1 = uniform_f64(b);
}

template <class E, int KIND>
__device__ __attribute__((noinline)) void run_node_task(int task_in, int flags_in) {
    using T = typename E::T;
    constexpr bool ACCEPT = KIND == kKindAcceptance;
    constexpr int METHOD = ACCEPT ? MPV_METHOD_SPECINFER : KIND;
    const Args& a = lds_launch().a;
    const Workspace& ws = lds_launch().ws;
    const QueuePlan& q = lds_launch().q;
    const TreeDesc& tree = g_tree;
    // (what arrives as an argument arrives in vector registers: back to scalar ones)
    int task = uniform_i32(task_in), flags = uniform_i32(flags_in);
    const int wave = uniform_i32(static_cast<int>(threadIdx.x) / kWave), lane = threadIdx.x & (kWave - 1);
    uint4* const lds_t = g_rows;
    uint4* const lds_d = g_rows + kLdsVecs * kTaskBlock;
    const int B = uniform_i32(a.B), N = uniform_i32(a.N), V = uniform_i32(a.V);
    const float k32 = uniform_f32(a.k32);
    const int member = uniform_i32(g_loop.team.member), team_size = uniform_i32(g_loop.team.size);

    // what a task number stands for (tree, node: made scalar explicitly, so that the table lookups
    // that follow have uniform addresses)
    struct NodeView { int b, n, k; bool resumed; size_t bn; const T* zt; const T* zd; };
    auto view_of = [&](int t) __attribute__((always_inline)) -> NodeView {
        NodeView v;
        v.resumed = t >= B * N + B;
        v.b = uniform_i32(v.resumed ? t - (B * N + B) : t / N);
        v.n = uniform_i32(v.resumed ? q.split_node : t % N);
        v.bn = static_cast<size_t>(v.b) * N + v.n;
        v.zt = uniform_ptr(static_cast<const T*>(a.zt)) + v.bn * V;
        v.zd = uniform_ptr(static_cast<const T*>(a.zd)) + v.bn * V;
        v.k = uniform_i32(tree.nchild[v.n]);
        return v;
    };

    // ---- the part of the pair this member keeps on chip while a task runs
    RetainedPart<E, kTaskBlock, kRegVecs, kLdsVecs> pair;
    // the children's tokens, their two logits and the uniforms, for the first wave's scalar steps
    __shared__ int ch_tok[MPV_MAX_CHILDREN];
    __shared__ float ch_zt[MPV_MAX_CHILDREN], ch_zd[MPV_MAX_CHILDREN];
    __shared__ float ch_u[MPV_MAX_CHILDREN + 1];      // last: the node's own uniform

    if (wave != 0) {
        // ---- a sweeping wave does what the first wave commands: it takes up a task (loads its
        //      share of the pair and runs the statistics sweep) or sweeps once more
        // what the second wave fetches of the children (kept as stored until the sweep is over)
        int pf_x = -1;
        float pf_u = 2.f;
        T pf_t = 0, pf_d = 0;
        int asked_for = -1;                               // the task whose rows this wave has asked for already
        // Asks for this wave's share of task t.  The second wave also fetches what the scalar steps
        // need of the children (lane j looks after child j): the tokens, then the two logits at each
        // token, and only then its row loads.  (Loads that depend on loads: issued after the row
        // loads they would wait for every one of them, the compiler cannot count past the
        // conditional ones; before them they wait for the tokens alone.)
        auto take_up = [&](int t) __attribute__((always_inline)) {
            const NodeView nv = view_of(t);
            pf_x = -1; pf_u = 2.f; pf_t = 0; pf_d = 0;
            if (wave == 1) {
                if (lane < nv.k && a.tokens) {
                    const size_t bc = static_cast<size_t>(nv.b) * N + tree.child_list[tree.child_off[nv.n] + lane];
                    pf_x = as_global(a.tokens)[bc];
                    if (!a.estimate) pf_u = as_global(a.uniforms)[bc];
                }
                if (lane == MPV_MAX_CHILDREN && !a.estimate) pf_u = as_global(a.uniforms)[nv.bn];
                if (pf_x >= 0 && pf_x < V) {
                    pf_t = as_global(nv.zt)[pf_x];
                    pf_d = as_global(nv.zd)[pf_x];
                }
            }
            int tid_l = threadIdx.x;
            asm volatile("" : "+v"(tid_l));     // per-task copy: nothing derived from it is kept across tasks
            pair.setup(nv.zt, nv.zd, V, lds_t, lds_d, tid_l, member, team_size, uniform_i32(q.part_vecs));
            pair.issue_loads();
            asked_for = t;
        };
        for (;;) {
            task_barrier();                                // B: the command is there
            const SweepCmd cmd = g_cmd;
            const int kind = uniform_i32(cmd.kind);
            if (kind == kCmdDone) {
                if (asked_for >= 0) wait_memory();        // (asked for in vain: nothing may land in LDS after this)
                return;
            }
            if (kind == kCmdTask) {
                const int t = uniform_i32(cmd.m);
                if (asked_for != t) take_up(t);
                asked_for = -1;
                const int kk = uniform_i32(tree.nchild[view_of(t).n]);
                PairStatsRawF<E> f;
                f.t.init(); f.d.init(); f.k32 = k32;
                pair.first_pass(f);
                if (wave == 1) {
                    if (lane < kk) { ch_tok[lane] = pf_x; ch_u[lane] = pf_u; ch_zt[lane] = E::load_one(&pf_t); ch_zd[lane] = E::load_one(&pf_d); }
                    if (lane == MPV_MAX_CHILDREN) ch_u[MPV_MAX_CHILDREN] = pf_u;
                }
                const float Mt_w = wave_max(f.t.mk), Md_w = wave_max(f.d.mk);
                const double st_w = wave_sum((f.t.s > 0.f) ? static_cast<double>(f.t.s * fast_exp2(f.t.mk - Mt_w)) : 0.0);
                const double sd_w = wave_sum((f.d.s > 0.f) ? static_cast<double>(f.d.s * fast_exp2(f.d.mk - Md_w)) : 0.0);
                if (lane == 0) {
                    g_sh.partf[wave][0] = Mt_w; g_sh.partf[wave][1] = Md_w;
                    g_sh.part[wave][0] = st_w; g_sh.part[wave][1] = sd_w;
                }
            } else {
                run_sweep<E, KIND>(pair, cmd, k32, wave, lane);
                const int nx = uniform_i32(cmd.next);
                if (nx >= 0) take_up(nx);                 // this wave's slots are free again: the next task's rows
            }
            task_barrier();                                // A: this wave's partial sums are there
        }
    }

    // ================================================================ the first wave
    Team team = uniform_struct(g_loop.team);           // in registers while the tasks run
    bool asked = uniform_i32(g_loop.asked) != 0;
    int own_task = -1, own_flags = 0;
    const bool leader = team.member == 0;
    const bool lead = leader && lane == 0;            // the one lane that talks to the rest of the launch
    // Takes a task up: the other waves are told, this wave's share of the pair is asked for.
    auto start_task = [&](const NodeView& v, int t) __attribute__((always_inline)) {
        if (lane == 0) { g_cmd.kind = kCmdTask; g_cmd.m = t; }
        task_barrier();                                    // B: the other waves take the task up
        int tid_l = threadIdx.x;
        asm volatile("" : "+v"(tid_l));     // per-task copy: nothing derived from it is kept across tasks
        pair.setup(v.zt, v.zd, V, lds_t, lds_d, tid_l, member, team_size, uniform_i32(q.part_vecs));
        pair.issue_loads();
    };
    // A task taken up before it was certain (the task this team is most likely to run next,
    // started while the leader still settles what follows from the last one), -1: none.
    int started = -1;
    // Outcomes settled by tasks that handed on to a child's task directly (see the end of the
    // task): published by the first task that goes the long way.  And the weight such a child
    // starts with (Traversal), known here without asking memory; negative: not known.
    unsigned long long chain_settled = 0ull, chain_accepted = 0ull;
    double a0_known = -1.0;
    // One node task after the other, for as long as the team knows its next one itself (the task
    // a node task hands to its own team: a child's, or the rest of the node where the tree
    // branches): no way back through the task loop, no queue in between.
    for (;;) {
    {
    const NodeView nv = view_of(task);
    const bool resumed = nv.resumed;
    const int b = nv.b, n = nv.n, k = nv.k;
    const size_t bn = nv.bn;
    const T* const zt = nv.zt;
    const T* const zd = nv.zd;
    (void)zt; (void)zd;
    own_task = -1; own_flags = 0;
    if (started != task) start_task(nv, task);            // (else: under way since the end of the task before)
    started = -1;
    double At_ = 0.0, Ad_ = 0.0, wa = 1.0;            // log2-partitions of the two rows; the node's weight
    int next_hint = -1;                               // goes out with a sweep command (SweepCmd::next)
    // one more sweep by all four waves; the team's sums come back
    auto sweep = [&](int kind, const ResidualConsts& rc, float sp, float sq, int m, int naive, double& s0, double& s1) __attribute__((always_inline)) {
        if (lane == 0) {
            g_cmd.kind = kind; g_cmd.nAt = rc.nAt; g_cmd.nAd = rc.nAd; g_cmd.rho = rc.rho;
            g_cmd.sp = sp; g_cmd.sq = sq; g_cmd.m = m; g_cmd.naive = naive; g_cmd.next = next_hint;
        }
        task_barrier();                                    // B
        SweepCmd cmd;
        cmd.kind = kind; cmd.nAt = uniform_f32(rc.nAt); cmd.nAd = uniform_f32(rc.nAd); cmd.rho = uniform_f32(rc.rho);
        cmd.sp = sp; cmd.sq = sq; cmd.m = m; cmd.naive = naive; cmd.next = -1;
        run_sweep<E, KIND>(pair, cmd, k32, 0, lane);
        task_barrier();                                    // A
        collect_sums(team, s0, s1);
    };
    // W(c) for one c
    auto residual_mass = [&](double cc) __attribute__((always_inline)) -> double {
        const ResidualConsts rc = cold_residual_consts(At_, Ad_, cc);
        double s0, s1;
        sweep(kCmdMass, rc, 0.f, 0.f, 0, 0, s0, s1);
        return uniform_f64(uniform_f64(rc.scale) * s0);
    };

    if (lead) atomicAdd(&a.counters[resumed ? MPV_COUNTER_NODE_TASKS_RESUMED : MPV_COUNTER_NODE_TASKS_RUN], 1u);
    // are teams idle?  Asked now, needed when this task hands on to the next (the leader's business)
    int idle_now = 0;
    if (lead) idle_now = ld_relaxed(&ws.qctl[4 + 2 * kMaxClasses]);
    const bool split_here = METHOD == MPV_METHOD_TRAVERSAL && a.lazy && !resumed && n == q.split_node;
    const bool idle_seen = (flags & kFlagIdle) != 0;

    // Traversal, only what is needed, and idle teams about: an only child's task is queued
    // now, ahead of its starting weight.  It reads its rows while this task reads its own and
    // then finds the weight published (or waits a moment for it), so that a chain of nodes
    // takes little more than one task's time.  If the weight turns out to be 0 it gives up.
    bool child_ahead = false;
    if (METHOD == MPV_METHOD_TRAVERSAL && a.lazy && k == 1 && !split_here && idle_seen) {
        const int cn = tree.child_list[tree.child_off[n]];
        if (tree.nchild[cn] > 0) {
            child_ahead = true;
            if (lead) append_task(tree, ws, tree.cls[cn], b * N + cn);
        }
    }

    // ---- softmax statistics of both rows: the one read of the pair from memory
    float un = 2.f;                                   // the node's own uniform
    {
        // Traversal: the starting weight comes from the parent's task, which published it
        // before it queued this task (or publishes it shortly, if this task was queued ahead).
        // The leader fetches it and passes it on with the statistics.  Value and "ready" flag
        // are one 64-bit word (a weight is never NaN), read and written with relaxed
        // device-scope atomics: no fence, no cache invalidation.  Asked for before the sweep:
        // the answer is there when the sweep is over.
        const bool wants_a0 = lead && METHOD == MPV_METHOD_TRAVERSAL && n != 0 && !(a0_known >= 0.0);
        unsigned long long bits = kNotReady;
        if (wants_a0) bits = ld_relaxed(reinterpret_cast<const unsigned long long*>(&ws.a0[bn]));
        PairStatsRawF<E> f;
        f.t.init(); f.d.init(); f.k32 = k32;
        pair.first_pass(f);
        double a0 = 1.0;
        if (wants_a0) {
            for (int spin = 0; spin < kMaxSpins && bits == kNotReady; ++spin) {
                if (wall_clock64() - team.t_start > kLaunchTimeoutTicks) break;
                __builtin_amdgcn_s_sleep(8);
                bits = ld_relaxed(reinterpret_cast<const unsigned long long*>(&ws.a0[bn]));
            }
            if (bits != kNotReady) {
                a0 = __longlong_as_double(static_cast<long long>(bits));
            } else {            // the parent's task never published it (must never happen): the subtree is written off
                a0 = 0.0;
                atomicAdd(&a.counters[MPV_COUNTER_DEPENDENCY_TIMEOUT], 1u);
            }
        }
        a0 = lane_f64(a0, 0);
        if (a0_known >= 0.0) a0 = a0_known;
        a0_known = -1.0;
        // lanes to their wave's largest reference, waves to the workgroup's, members to the team's
        const float Mt_w = wave_max(f.t.mk), Md_w = wave_max(f.d.mk);
        const double st_w = wave_sum((f.t.s > 0.f) ? static_cast<double>(f.t.s * fast_exp2(f.t.mk - Mt_w)) : 0.0);
        const double sd_w = wave_sum((f.d.s > 0.f) ? static_cast<double>(f.d.s * fast_exp2(f.d.mk - Md_w)) : 0.0);
        if (lane == 0) {
            g_sh.partf[0][0] = Mt_w; g_sh.partf[0][1] = Md_w;
            g_sh.part[0][0] = st_w; g_sh.part[0][1] = sd_w;
        }
        task_barrier();                                    // A: every wave's partials are there
        un = ch_u[MPV_MAX_CHILDREN];
        team.seq++;
        float Mt = g_sh.partf[0][0], Md = g_sh.partf[0][1];
#pragma unroll
        for (int w = 1; w < kTaskWaves; ++w) { Mt = fmaxf(Mt, g_sh.partf[w][0]); Md = fmaxf(Md, g_sh.partf[w][1]); }
        double st = 0.0, sd = 0.0;
#pragma unroll
        for (int w = 0; w < kTaskWaves; ++w) {
            st += g_sh.part[w][0] * static_cast<double>(fast_exp2(g_sh.partf[w][0] - Mt));
            sd += g_sh.part[w][1] * static_cast<double>(fast_exp2(g_sh.partf[w][1] - Md));
        }
        unsigned mine = 0u;
        switch (lane) {
            case 0: mine = __float_as_uint(Mt); break;
            case 1: mine = __float_as_uint(Md); break;
            case 2: mine = half_of(st, 0); break;
            case 3: mine = half_of(st, 1); break;
            case 4: mine = half_of(sd, 0); break;
            case 5: mine = half_of(sd, 1); break;
            case 6: mine = half_of(a0, 0); break;
            case 7: mine = half_of(a0, 1); break;
            default: break;
        }
        exchange_words(team, mine);
        __builtin_amdgcn_wave_barrier();
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        team.dead = g_sh.dead;
        float MT = OnlineLse::kFloor, MD = OnlineLse::kFloor;
        for (int m = 0; m < team.size; ++m) {
            MT = fmaxf(MT, __uint_as_float(g_sh.words[m * kExchWords]));
            MD = fmaxf(MD, __uint_as_float(g_sh.words[m * kExchWords + 1]));
        }
        double ST = 0.0, SD = 0.0;
        for (int m = 0; m < team.size; ++m) {
            ST += double_at(g_sh.words, m, 1) * static_cast<double>(fast_exp2(__uint_as_float(g_sh.words[m * kExchWords]) - MT));
            SD += double_at(g_sh.words, m, 2) * static_cast<double>(fast_exp2(__uint_as_float(g_sh.words[m * kExchWords + 1]) - MD));
        }
        const double lg = cold_log2(lane == 1 ? SD : ST);         // both logarithms in one go, a lane each
        At_ = uniform_f64(static_cast<double>(MT) + lane_f64(lg, 0));
        Ad_ = uniform_f64(static_cast<double>(MD) + lane_f64(lg, 1));
        if (METHOD == MPV_METHOD_TRAVERSAL) wa = uniform_f64(double_at(g_sh.words, 0, 3));
    }
    RowStat rt, rd;
    rt.A = At_; rd.A = Ad_; rt.m = 0.f; rd.m = 0.f;

    // ---- per-child scalars and one residual-mass reduction per child
    if (METHOD == MPV_METHOD_TRAVERSAL && a.lazy && n != 0 && !(wa > 0.0) && chain_settled == 0ull) {
        // queued ahead of its weight, which is 0: the parent has written off the whole subtree.
        // Nothing to do but to pass the news on to an only child queued ahead in turn.
        if (lead) {
            if (child_ahead) {
                const size_t bc = static_cast<size_t>(b) * N + tree.child_list[tree.child_off[n]];
                st_relaxed(reinterpret_cast<unsigned long long*>(&ws.a0[bc]), static_cast<unsigned long long>(__double_as_longlong(0.0)));
            }
            wait_memory();
            atomicAdd(&ws.qctl[1], 1);
        }
        goto task_end;
    }
    double c = 0.0, W = 1.0;
    const double kd = static_cast<double>(k32);
    // p(x) and q(x) of every child's token at once: lane j has the target's, lane 32 + j the draft's
    static_assert(MPV_MAX_CHILDREN <= 32, "one lane per child and row");
    double pq_all;
    {
        const int j = lane & 31;
        const bool of_draft = lane >= 32;
        const float z = j < k ? (of_draft ? ch_zd[j] : ch_zt[j]) : 0.f;
        pq_all = probability_exp2(static_cast<double>(z) * kd - (of_draft ? Ad_ : At_));
    }
    // test outcomes this task settles, one bit per node at its position in postorder
    unsigned long long settled_bits = 0ull, accepted_bits = 0ull;
    int next_node = -1;                               // SpecInfer, only what is needed: the accepted child
    double own_w = 0.0;                               // ... and the weight it starts with
    int own_child = -1;                               // Traversal: index of the first child whose task is to be run
    bool paused = false;
    bool own_given = false;                           // that child's task was queued after all (some team is idle)
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
            const ResidualConsts rc = cold_residual_consts(rt.A, rd.A, x);
            double sum_w, sum_q;
            sweep(kCmdMassSlope, rc, 0.f, 0.f, 0, 0, sum_w, sum_q);
            const double scale = uniform_f64(rc.scale);
            const double Wx = uniform_f64(scale * sum_w);
            const double dWx = -uniform_f64(scale * sum_q) / x;       // the sweep added up rho q over {p > rho q}
            const double Dx = fmin(fmax((Wx + x - 1.0) / x, 0.0), 1.0);
            const double dDx = (dWx + 1.0 - Dx) / x;
            const double kk = static_cast<double>(k);
            fx = Wx - int_power(Dx, k);
            dfx = dWx - kk * int_power(Dx, k - 1) * dDx;
            sp_rho = x;
            sp_W = Wx;
            if (team.dead) break;
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
        // (nothing follows from such a task: the team asks for its next one right away)
        if (leader && !asked) {
            if (lane == 0) st_relaxed(&ws.mailbox[team.id], kMailboxSoon);
            asked = true;
        }
        double alpha;
        if (a.walk == 3) {
            const double D = fmin(fmax((sp_W + sp_rho - 1.0) / sp_rho, 0.0), 1.0);
            alpha = 1.0 - int_power(D, k);
        } else if (a.walk == 0) {
            double cc = 0.0, Wc = 1.0;
            for (int j = 0; j < k && Wc > 0.0 && !team.dead; ++j) {
                cc = uniform_f64(cc + Wc);
                Wc = residual_mass(cc);
            }
            alpha = 1.0 - Wc;
        } else {
            const float At_hi = static_cast<float>(rt.A), Ad_hi = static_cast<float>(rd.A);
            ResidualConsts rc;
            rc.nAt = -At_hi; rc.nAd = -Ad_hi; rc.rho = 0.f; rc.scale = 1.0;
            double s0, s1;
            sweep(kCmdAcceptance, rc, static_cast<float>(cold_exp2(static_cast<double>(At_hi) - rt.A)),
                  static_cast<float>(cold_exp2(static_cast<double>(Ad_hi) - rd.A)), a.walk == 1 ? k : k - 1, a.walk == 2 ? 1 : 0, s0, s1);
            alpha = s0;
        }
        // the answer may be there already: then the team goes straight on (see the end of the other tasks)
        if (leader && asked && !team.dead) {
            const int previous = uniform_i32(g_loop.previous_task);
            int t = -1;
            if (lane == 0) t = ld_relaxed(&ws.mailbox[team.id]);
            t = uniform_i32(t);
            if (t >= 0 && t != previous) {
                asked = false;
                if (lane == 0) g_loop.previous_task = t;
                team_announce(team, t, 0);
                if (!(t >= B * N && t < B * N + B)) {
                    start_task(view_of(t), t);
                    started = t;
                }
                own_task = t;                              // (announced; counted when it was queued)
            }
        }
        if (lead) {
            as_global(a.alpha)[bn] = static_cast<float>(fmin(fmax(alpha, 0.0), 1.0));
            atomicAdd(&ws.qctl[1], 1);
        }
        goto task_end;
    }
    for (int j = 0; j < k; ++j) {
        // a resumed task repeats the arithmetic of the first child (whose task has long run)
        // to get at the residual that follows its rejection
        const bool redone = resumed && j == 0;
        const int cn = tree.child_list[tree.child_off[n] + j];
        const size_t bc = static_cast<size_t>(b) * N + cn;
        const int x = ch_tok[j];
        double px = 0.0, qx = 0.0;
        const bool tok_ok = (x >= 0 && x < V);
        if (tok_ok) {
            px = lane_f64(pq_all, j);
            qx = lane_f64(pq_all, 32 + j);
        } else if (lead) {
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
            // kept for this team if it is the last thing this task finds out and nobody is idle
            own_child = j;
            own_w = w_child;
            own_given = (idle_seen || j < k - 1 || child_ahead) && !(split_here && j == 0);
        }
        // One more sweep to go at most: time to ask for the next task, unless this team
        // already knows what it will run next (a child's task).
        if (leader && j == k - 1 && !asked && (own_child < 0 || own_given) &&
            !(METHOD == MPV_METHOD_SPECINFER && a.lazy && child_accepted && tree.nchild[cn] > 0)) {
            if (lane == 0) st_relaxed(&ws.mailbox[team.id], kMailboxSoon);
            asked = true;
        }
        if (lead && !redone) {
            if (METHOD == MPV_METHOD_TRAVERSAL) {
                if (tree.nchild[cn] == 0) {
                    st_shared_f64(&ws.atest[bc], w_child);           // leaves are tested as they are
                } else {
                    st_relaxed(reinterpret_cast<unsigned long long*>(&ws.a0[bc]), static_cast<unsigned long long>(__double_as_longlong(w_child)));
                    // The first child that needs a task is kept for this team (run next,
                    // no queue) unless some team is idle; every other one is queued now,
                    // while this task goes on with the sweeps that follow.
                    if (run_child && (!first_to_run || own_given) && !child_ahead)
                        append_task(tree, ws, tree.cls[cn], b * N + cn);      // (waits for the weight's store with its own count)
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
                as_global(a.dbg_edge)[bc * 2] = static_cast<float>(px);
                as_global(a.dbg_edge)[bc * 2 + 1] = static_cast<float>(qx);
            }
        }

        // Where the tree branches and no team is to spare, the first child's subtree is
        // explored first: most walks end there, and then nothing else of this node is needed.
        if (split_here && j == 0 && run_child) {
            paused = true;
            break;
        }

        if (METHOD == MPV_METHOD_SPECINFER && a.walk >= 2 && !a.estimate && lead &&
            fabs(w_child - static_cast<double>(ch_u[j])) < 1e-6)
            atomicAdd(&a.counters[MPV_COUNTER_NEAR_TIE_ACCEPT], 1u);     // (the other rules count these in their walk)
        // SpecInfer moves into the first child it accepts: later children and this node's
        // residual are not needed (the same in every lane: no lane is left behind)
        if (METHOD == MPV_METHOD_SPECINFER && a.lazy && child_accepted) {
            next_node = cn;
            if (a.context_node) {
                // the walk goes on at the node of the accepted entry's context (anything else than a node
                // number is ignored)
                const int stands_for = uniform_i32(as_global(a.context_node)[static_cast<size_t>(b) * N + cn]);
                if (stands_for >= 0 && stands_for < N) next_node = stands_for;
            }
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
        if (team.dead) break;
        const double c2 = uniform_f64(c + W / wa);
        // the task's last sweep, and the team goes on with a child's task: the other waves may ask for its rows
        if (METHOD == MPV_METHOD_TRAVERSAL && j == k - 1 && own_child >= 0 && !own_given)
            next_hint = b * N + tree.child_list[tree.child_off[n] + own_child];
        const double W2 = residual_mass(c2);
        next_hint = -1;
        if (W2 > 0.0) {
            if (METHOD == MPV_METHOD_TRAVERSAL) {
                const double S = (wa / W) * W2;
                wa = uniform_f64(S / (S + (1.0 - wa)));
            }
            c = c2;
            W = W2;
        } else {
            if (METHOD == MPV_METHOD_TRAVERSAL) wa = (wa >= 1.0) ? 1.0 : 0.0;
            if (lead) atomicAdd(&a.counters[MPV_COUNTER_ZERO_MASS], 1u);
        }
        if (METHOD == MPV_METHOD_SPECINFER && a.walk == 2) {
            // Naive, estimate (App. D, Naive Branching): p_res(x_i) for every child, p_res = norm (p - q)_+
            // (now c = 1 and W = its mass; p itself if the mass was zero: c = 0, W = 1)
            for (int i = 0; i < k; ++i) {
                const int ci = tree.child_list[tree.child_off[n] + i];
                const int xi = ch_tok[i];
                double r = 0.0;
                if (xi >= 0 && xi < V)
                    r = fmax(lane_f64(pq_all, i) - c * lane_f64(pq_all, 32 + i), 0.0) / W;
                else if (i > 0 && lead)
                    atomicAdd(&a.counters[MPV_COUNTER_BAD_TOKEN], 1u);
                if (lead) {
                    st_shared_f64(&ws.aux[static_cast<size_t>(b) * N + ci], r);
                    if (i > 0) st_shared_f64(&ws.atest[static_cast<size_t>(b) * N + ci], 0.0);   // never tested
                }
                settled_bits |= 1ull << tree.rank[ci];
            }
            break;
        }
    }

    // ---- The sweeps are over and the part on chip is no longer needed.  What this team will
    //      most likely run next (every member works it out by itself, from the same numbers) is
    //      taken up at once: its rows travel while the leader settles what follows from this
    //      task, and while the others wait to hear of it.
    int likely = -1;
    if (!team.dead) {
        if (METHOD == MPV_METHOD_TRAVERSAL) {
            if (paused) likely = b * N + tree.child_list[tree.child_off[n]];
            else if (own_child >= 0 && !own_given) likely = b * N + tree.child_list[tree.child_off[n] + own_child];
        } else if (a.lazy && next_node >= 0 && tree.nchild[next_node] > 0) {
            likely = b * N + next_node;
        }
    }
    // The team has asked for its next task ahead of time; if the answer is in the mailbox already
    // (and nothing of this task's own can come first) the team is told now and takes the task
    // up, while the leader settles what follows from this one: whatever that produces then goes
    // to the queue instead of being run by this team.  (Not where the branching node may have to
    // be resumed: that task has no place in the queue.  Nor with the token-following rules: a
    // tree can need several draws, the queue has room for one.)
    int taken = -1;
    if (leader && likely < 0 && !paused && asked && !team.dead && a.walk == 0 &&
        !(METHOD == MPV_METHOD_TRAVERSAL && a.lazy && q.split_node >= 0)) {
        const int previous = uniform_i32(g_loop.previous_task);
        int t = -1;
        if (lane == 0) t = ld_relaxed(&ws.mailbox[team.id]);
        t = uniform_i32(t);
        if (t >= 0 && t != previous) {
            taken = t;
            asked = false;
            if (lane == 0) g_loop.previous_task = t;
            team_announce(team, t, uniform_i32(idle_now) != 0 ? kFlagIdle : 0);
        }
    }
    {
        const int start_now = likely >= 0 ? likely : ((taken >= 0 && !(taken >= B * N && taken < B * N + B)) ? taken : -1);
        if (start_now >= 0) {
            start_task(view_of(start_now), start_now);
            started = start_now;
        }
        if (likely >= 0) {
            // Where that task is a child's and nothing else follows from this one (a chain), the
            // team simply goes on with it: every member knows the task and what it starts with,
            // so nothing is announced, nothing waited for, and the outcomes settled here are
            // noted for the first task that goes the long way to publish.  (If another branch
            // settles the tree meanwhile, the chain runs on in vain until it ends.)
            if (METHOD == MPV_METHOD_TRAVERSAL || a.walk == 0) {
                if (!(METHOD == MPV_METHOD_TRAVERSAL && paused)) {
                    if (lead) {
                        st_shared_f64(&ws.At[bn], rt.A);
                        st_shared_f64(&ws.Ad[bn], rd.A);
                        st_shared_f64(&ws.cfin[bn], c);
                        if (METHOD == MPV_METHOD_TRAVERSAL && n != 0) st_shared_f64(&ws.atest[bn], wa);
                    }
                    chain_settled |= settled_bits;
                    chain_accepted |= accepted_bits;
                    if (METHOD == MPV_METHOD_TRAVERSAL && n != 0) {
                        const unsigned long long own = 1ull << tree.rank[n];
                        chain_settled |= own;
                        if (static_cast<double>(un) < wa) chain_accepted |= own;
                    }
                }
                if (METHOD == MPV_METHOD_TRAVERSAL) a0_known = own_w;
                task = likely;                            // (flags: as they are)
                continue;
            }
        }
    }
    settled_bits |= chain_settled;
    accepted_bits |= chain_accepted;
    chain_settled = 0ull;
    chain_accepted = 0ull;

    // ---- what follows from this task: the leader's business (its first wave's)
    if (!leader) goto task_end;
    own_flags = uniform_i32(idle_now) != 0 ? kFlagIdle : 0;
    if (paused) {
        // nothing is settled yet; the first child's task is run next by this team
        own_task = b * N + tree.child_list[tree.child_off[n]];
        team_announce(team, own_task, own_flags);
        if (lane == 0) {
            (void)atomicAdd(&ws.qctl[0], 1);
            wait_memory();                            // counted (and the child's weight written) before this task counts as finished
            atomicAdd(&ws.qctl[1], 1);
        }
        goto task_end;
    }
    int push_sample_i = 0, settled_i = 0, resume_i = 0;
    if (lane == 0) {
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
                if (static_cast<double>(un) < wa) accepted_bits |= own;
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
                const unsigned long long all = (N >= 64) ? ~0ull : ((1ull << N) - 1ull);
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
        push_sample_i = push_sample ? 1 : 0;
        settled_i = settled_tree ? 1 : 0;
        resume_i = resume ? 1 : 0;
    }
    push_sample_i = uniform_i32(push_sample_i);
    settled_i = uniform_i32(settled_i);
    resume_i = uniform_i32(resume_i);
    // What follows from this task.  One task is run by this team itself, next (no queue,
    // no waiting): the sampling if this task settled the tree, else the first child that needs
    // its own task (Traversal) or the accepted child (SpecInfer).  The other children are queued.
    if (push_sample_i) {
        if (!ACCEPT && a.estimate) {
            // the expected block efficiency instead of a walk: scalar work over the tree's
            // per-node results, done here and now by this wave (there are no uniforms to walk with)
            estimate_wave<METHOD>(tree, ws, a, b);
        } else if (taken >= 0) {
            if (lane == 0) append_task(tree, ws, 0, B * N + b);      // (the results were waited for above)
        } else {
            own_task = B * N + b;
        }
    } else if (taken >= 0) {
        // (nothing else can follow from a task that has no child of its own to run)
    } else if (resume_i) {
        own_task = B * N + B + b;
    } else if (METHOD == MPV_METHOD_TRAVERSAL) {
        if (own_child >= 0 && !own_given && !settled_i) own_task = b * N + tree.child_list[tree.child_off[n] + own_child];
    } else if (a.lazy && next_node >= 0 && tree.nchild[next_node] > 0) {
        own_task = b * N + next_node;
    }
    // the others hear of it at once (they are waiting for the next task by now)
    if (own_task >= 0) team_announce(team, own_task, own_flags);
    if (lane == 0) {
        if (own_task >= 0) {
            (void)atomicAdd(&ws.qctl[0], 1);
            wait_memory();
        }
        // (cannot happen: a task that settles the tree or completes a subtree has no child left to run)
        if (METHOD == MPV_METHOD_TRAVERSAL && own_child >= 0 && !own_given && !settled_i && (push_sample_i || resume_i)) {
            const int cn = tree.child_list[tree.child_off[n] + own_child];
            append_task(tree, ws, tree.cls[cn], b * N + cn);
        }
        wait_memory();                                // every new task has been counted
        atomicAdd(&ws.qctl[1], 1);
    }
    if (taken >= 0) own_task = taken;                 // (announced above; counted when it was queued)
    }   // (the task's own scope)
task_end:
    // The task that follows: the leader knows (and has told the others, who hear of it here).
    int next, next_flags = 0;
    if (leader) {
        next = own_task;
        next_flags = own_flags;
    } else {
        next = team_listen(team, next_flags, ws);
    }
    const bool node_next = next >= 0 && !(next >= B * N && next < B * N + B) && !team.dead;
    if (started >= 0 && (!node_next || next != started)) {
        // taken up in vain (the tree was settled meanwhile, or the task went elsewhere): the other
        // waves finish their sweep, this wave's loads land, and the slots are free again
        task_barrier();                                    // A
        wait_memory();
        started = -1;
    }
    if (!node_next) {
        if (lane == 0) g_cmd.kind = kCmdDone;
        task_barrier();                                    // B: the other waves leave
        if (lane == 0) {
            g_loop.team = team;
            g_loop.asked = asked ? 1 : 0;
            g_loop.own_task = next;                       // (already announced to, or heard by, the team)
            g_loop.own_flags = next_flags;
        }
        return;
    }
    task = next;
    flags = next_flags;
    }   // node tasks
}


// (disable_tail_calls: a call marked as a possible tail call makes the compiler treat the callee
// as one that must preserve registers for its caller, and the task functions, which use nearly
// all of them, would save and restore dozens per call in private memory)
template <class E, int KIND>
__global__ __launch_bounds__(kTaskBlock) __attribute__((amdgpu_waves_per_eu(3, 3))) __attribute__((disable_tail_calls))
void node_task_kernel(const Launch* __restrict__ launch) {
    // KIND: MPV_METHOD_SPECINFER (all top-down rules) or MPV_METHOD_TRAVERSAL, or kKindAcceptance: the
    // top-down kernel reduced to what the acceptance rates need (an instantiation of its own, so that
    // its extra sweeps do not weigh on the register allocation of the verification kernels)
    constexpr bool ACCEPT = KIND == kKindAcceptance;
    constexpr int METHOD = ACCEPT ? MPV_METHOD_SPECINFER : KIND;
    __shared__ int sh_task, sh_flags;
    // The launch parameters and the tree tables are read from LDS, copied there from the
    // workspace (init_kernel put them there): as kernel arguments, handed on by reference or
    // indexed with a value the compiler keeps in a vector register, they were copied, whole,
    // into every lane's private memory.
    for (int w = threadIdx.x; w < static_cast<int>(sizeof(Launch) / sizeof(int)); w += kTaskBlock)
        g_launch_words[w] = reinterpret_cast<const int*>(launch)[w];
    for (int w = threadIdx.x; w < static_cast<int>(sizeof(TreeDesc) / sizeof(int)); w += kTaskBlock)
        reinterpret_cast<int*>(&g_tree)[w] = reinterpret_cast<const int*>(launch->ws.tree)[w];
    __syncthreads();
    const QueuePlan& q = lds_launch().q;
    const Workspace& ws = lds_launch().ws;
    const Args& a = lds_launch().a;
    const TreeDesc& tree = g_tree;                // the task loop starts with a barrier

    // ---- this workgroup's place in its team
    const bool drop_settled = METHOD == MPV_METHOD_TRAVERSAL && a.lazy != 0;
    const int wave = uniform_i32(static_cast<int>(threadIdx.x) / kWave);
    bool leader;
    {
        Team team;
        team.size = q.team_size;
        const int i = static_cast<int>(blockIdx.x);
        if (q.same_xcd) {                         // workgroup i runs on chiplet i % 8: keep a team on one
            const int r = i / 8;
            team.id = (i % 8) + 8 * (r / team.size);
            team.member = r % team.size;
        } else {
            team.id = i / team.size;
            team.member = i % team.size;
        }
        team.seq = 0u; team.tseq = 0u; team.dead = 0;
        team.area = ws.exch + static_cast<size_t>(team.id) * 2 * team.size * kExchWords;
        team.task_word = ws.team_task + static_cast<size_t>(team.id) * 2;
        team.t_start = wall_clock64();
        leader = team.member == 0;
        if (threadIdx.x == 0) {
            g_loop.team = team;
            g_loop.asked = 1;                     // the team starts out waiting
            g_loop.own_task = leader ? -1 : kNothingHeard;
            g_loop.own_flags = 0;
            g_loop.previous_task = -4;            // none yet
            // the last member to arrive opens the team's mailbox: from then on the dispatcher may hand it tasks
            const int n_arrived = atomicAdd(&ws.arrived[team.id], 1) + 1;
            if (n_arrived == team.size) st_relaxed(&ws.mailbox[team.id], kMailboxWaiting);
        }
    }
    // The first wave's scalar steps are the critical path of every task and few in number: they
    // go first when the compute unit's waves compete for issue slots.
    if (wave == 0) __builtin_amdgcn_s_setprio(3);
    for (;;) {
    __syncthreads();                                  // the previous task is done with LDS; g_loop is as it left it
    if (wave == 0) {
        // the task loop's own state: taken from g_loop, put back before the barrier below
        Team team = uniform_struct(g_loop.team);
        bool asked = uniform_i32(g_loop.asked) != 0;
        int own_task = uniform_i32(g_loop.own_task), own_flags = uniform_i32(g_loop.own_flags);
        int previous_task = uniform_i32(g_loop.previous_task);
        int task = kTaskExit, flags = 0;
        if (team.dead) {
            task = kTaskExit;
        } else if (leader) {
            for (;;) {
                if (own_task >= 0) {
                    task = own_task;
                    flags = own_flags;
                    own_task = -1;
                    break;
                }
                if (!asked) {
                    if (threadIdx.x == 0) st_relaxed(&ws.mailbox[team.id], kMailboxWaiting);
                    wait_memory();
                }
                task = acquire_task(team.id, previous_task, drop_settled, team.t_start);
                // are teams idle (as of the last round of dispatching)?
                flags = uniform_i32(ld_relaxed(&ws.qctl[4 + 2 * kMaxClasses])) != 0 ? kFlagIdle : 0;
                previous_task = task;
                asked = false;
                // tasks without any V-wide work are the leader's alone; everything else is announced
                const bool solo = task != kTaskExit && task >= a.B * a.N && task < a.B * a.N + a.B && (ACCEPT || a.estimate);
                if (solo) {
                    if (!ACCEPT) estimate_wave<METHOD>(tree, ws, a, task - a.B * a.N);
                    if (threadIdx.x == 0) {
                        wait_memory();
                        atomicAdd(&ws.qctl[1], 1);
                    }
                    continue;
                }
                team_announce(team, task, flags);
                break;
            }
        } else if (own_task != kNothingHeard) {
            task = own_task;
            flags = own_flags;
            own_task = kNothingHeard;
        } else {
            task = team_listen(team, flags, ws);
        }
        const bool sampling = task != kTaskExit && task >= a.B * a.N && task < a.B * a.N + a.B && !(ACCEPT || a.estimate);
        if (sampling && leader && !asked) {
            // the walk and the bonus token come next: one sweep or two, then the team is free
            if (threadIdx.x == 0) st_relaxed(&ws.mailbox[team.id], kMailboxSoon);
            asked = true;
        }
        if (threadIdx.x == 0) {
            g_loop.team = team;
            g_loop.asked = asked ? 1 : 0;
            g_loop.own_task = own_task;
            g_loop.own_flags = own_flags;
            g_loop.previous_task = previous_task;
            sh_task = task; sh_flags = flags;
        }
    }
    __syncthreads();
    const int task = uniform_i32(sh_task), flags = uniform_i32(sh_flags);
    if (task == kTaskExit) break;
    if (task >= a.B * a.N && task < a.B * a.N + a.B) {
        if (ACCEPT || a.estimate) {
            // no walk in these modes (there are no uniforms): scalar work of the leader's first
            // wave alone, whichever way the task came
            if (wave == 0 && leader) {
                if (!ACCEPT) estimate_wave<METHOD>(tree, ws, a, task - a.B * a.N);
                if (threadIdx.x == 0) {
                    wait_memory();
                    atomicAdd(&ws.qctl[1], 1);
                }
            }
            continue;
        }
        // the tree's outcome is settled: walk and bonus token
        const int next = sample_task<E, METHOD>(task - a.B * a.N);
        if (wave == 0 && leader) {
            if (next >= 0) {                          // a token-following walk goes on
                Team team = uniform_struct(g_loop.team);          // (as sample_task left it)
                team_announce(team, next, flags);
                if (threadIdx.x == 0) {
                    g_loop.team = team;
                    g_loop.own_task = next;
                    g_loop.own_flags = flags;
                }
            }
            if (threadIdx.x == 0) {
                if (next >= 0) {
                    (void)atomicAdd(&ws.qctl[0], 1);
                    wait_memory();                    // counted (and the walk's position written) first
                }
                atomicAdd(&ws.qctl[1], 1);
            }
        }
        continue;
    }
    run_node_task<E, KIND>(task, flags);
    }   // task loop
}

// ------------------------------------------------------------------ walk
//
// The uniform-dependent part of SpecInfer and Traversal, run by the first wave of every member of
// the sampling team (they all need the stopping node; the leader records the path): lane n compares u[n] with the probability node n is tested with
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
    as_global(a.accept_len)[b] = len;
    int32_t* pn = a.path_nodes + static_cast<size_t>(b) * a.max_depth;
    int32_t* pt = a.path_tokens + static_cast<size_t>(b) * a.max_depth;
    for (int i = len; i < a.max_depth; ++i) { pn[i] = -1; pt[i] = -1; }
    for (int n = stop, i = len - 1; n > 0; n = tree.parent[n], --i) {
        pn[i] = n;
        pt[i] = as_global(a.tokens)[base + n];
    }
}

template <int METHOD>
__device__ __forceinline__ int walk_wave(const TreeDesc& tree, const Workspace& ws, const Args& a, int b, bool record) {
    const int lane = threadIdx.x & (kWave - 1);
    const size_t base = static_cast<size_t>(b) * a.N;
    bool acc = false, near = false;
    if (lane > 0 && lane < a.N) {
        const double at = ld_shared_f64(&ws.atest[base + lane]);
        const double uu = static_cast<double>(as_global(a.uniforms)[base + lane]);
        acc = uu < at;
        near = fabs(at - uu) < 1e-6;
        if (a.dbg_accept && record) as_global(a.dbg_accept)[base + lane] = static_cast<float>(at);
    }
    if (lane == 0 && a.dbg_accept && record) as_global(a.dbg_accept)[base] = 1.f;
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
    if (lane == 0 && record) {
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
            const int x = as_global(a.tokens)[base + n];
            double none_before = 1.0, none_at_all = 1.0;
            bool first_carrier = true;
            int j = 0;
            // trees of distinct contexts, SpecTr: an accepted entry leads to the node it stands for, so a
            // node collects the acceptances of every entry that stands for it and a repeat collects nothing
            const bool aliased = a.walk == 3 && a.context_node != nullptr;
            double through_entries = 0.0;
            for (int l = 0; l < k; ++l) {
                const int sib = tree.child_list[off + l];
                if (sib == n) j = l;
                if (sib < n) {                        // list order is node order
                    none_before *= 1.0 - sh_v[sib];
                    if (as_global(a.tokens)[base + sib] == x) first_carrier = false;
                }
                if (aliased && as_global(a.context_node)[base + sib] == n) through_entries += sh_v[sib] * none_at_all;
                none_at_all *= 1.0 - sh_v[sib];
            }
            if (a.walk == 0) step = sh_v[n] * none_before;
            else if (a.walk == 1) step = first_carrier ? sh_v[n] : 0.0;
            else if (a.walk == 2) {
                const double a1 = sh_v[tree.child_list[off]];
                step = (j == 0 ? a1 : 0.0) + (first_carrier ? (1.0 - a1) * sh_w[n] : 0.0);
            } else if (aliased) {
                step = through_entries + (first_carrier ? sh_w[n] * none_at_all : 0.0);
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
    if (live && a.reach_prob) as_global(a.reach_prob)[base + n] = static_cast<float>(reach);
    const double total = wave_sum(live ? reach : 0.0);
    if (n == 0 && a.expected) as_global(a.expected)[b] = static_cast<float>(total);
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
                r[i] = (e < V) ? term(E::load_one_global(zt + e), use_d ? E::load_one_global(zd + e) : 0.f) : 0.f;
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


// tile_sum: kMaxTiles floats of LDS.  Everything it reads from the workspace was written by node
// tasks of this launch (see st_shared_f64) before the task that started this one was announced.
// The vocabulary is split among the members in runs of whole wave tiles, in member order; each
// member adds up the masses of its tiles, one exchange gives everybody every member's total, and
// the member whose run contains u * R finds the token.
template <class E, int METHOD>
__device__ __attribute__((noinline)) int sample_task(int b_in) {
    using T = typename E::T;
    const Args& a = lds_launch().a;
    const Workspace& ws = lds_launch().ws;
    const TreeDesc& tree = g_tree;
    const int b = uniform_i32(b_in);
    float* const tile_sum = reinterpret_cast<float*>(g_rows);
    Team team = uniform_struct(g_loop.team);           // every lane its copy; they stay alike
    struct WriteBack {                                 // (after the function's last barrier: nobody reads the old one any more)
        Team& t;
        __device__ ~WriteBack() { if (threadIdx.x == 0) g_loop.team = t; }
    } write_back{team};
    constexpr int NW = kTaskWaves;
    constexpr int PER_LANE = ResidualTile<E>::PER_LANE;
    constexpr int TILE = ResidualTile<E>::TILE;
    __shared__ int sh_tile;
    __shared__ double sh_before, sh_local_total;

    __shared__ int sh_stop, sh_next;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const bool leader = team.member == 0;
    const bool lead = leader && threadIdx.x == 0;
    if (wave == 0) {
        // where the token is drawn: the node the rule stops in, or the node a token-following
        // walk has reached
        const int stop = a.walk ? ld_relaxed(&ws.cur[b]) : walk_wave<METHOD>(tree, ws, a, b, leader);
        if (lane == 0) { sh_stop = stop; sh_next = -1; }
    }
    __syncthreads();
    const int n = __builtin_amdgcn_readfirstlane(sh_stop);
    const size_t bn = static_cast<size_t>(b) * a.N + n;
    const T* zt = static_cast<const T*>(a.zt) + bn * a.V;
    const T* zd = static_cast<const T*>(a.zd) + bn * a.V;
    const int V = a.V;
    const int ntiles = (V + TILE - 1) / TILE;
    // this member's run of tiles
    const int per = (ntiles + team.size - 1) / team.size;
    const int t_lo = min(team.member * per, ntiles), t_hi = min(t_lo + per, ntiles);
    const int my_tiles = t_hi - t_lo;

    double At, Ad = 0.0, c = 0.0;
    if (tree.nchild[n] == 0 || a.walk == 1) {
        // a leaf (its target row has not been touched yet) or an NSS draw: from p itself
        RowStatsF<E> f;
        f.t.init(); f.k32 = a.k32;
        const int e_lo = t_lo * TILE, e_hi = min(V, t_hi * TILE);
        if (e_hi > e_lo) sweep_row<E, kTaskBlock, 2 * kTaskUnroll>(zt + e_lo, e_hi - e_lo, f);
        OnlineLse none; none.init();
        double unused_d, unused_a0;
        __shared__ double sh_no_weight;
        if (threadIdx.x == 0) sh_no_weight = 0.0;
        team_stats(team, f.t, none, &sh_no_weight, At, unused_d, unused_a0);
        if (lead) ws.At[bn] = At;
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

    // ---- pass 1: mass of every wave tile of this member's run, in vocabulary order
    //      (tile_sum[i] belongs to tile t_lo + i)
    {
        // Whole, aligned tiles are taken U at a time per wave with all their loads issued
        // before the first use.
        int t_next = t_lo + wave;
        constexpr int U = 8;
        const int whole = min(rt_.aligned ? V / TILE : 0, t_hi);
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
                for (int j = 0; j < U; ++j) tile_sum[t_next + j * NW - t_lo] = s[j];
            }
        }
        for (int t = t_next; t < t_hi; t += NW) {
            float r[PER_LANE];
            rt_.load(t, lane, r);
            float ls = 0.f;
#pragma unroll
            for (int i = 0; i < PER_LANE; ++i) ls += r[i];
            const float w = wave_sum_f32(ls);
            if (lane == 0) tile_sum[t - t_lo] = w;
        }
    }
    __syncthreads();

    // ---- this member's total (wave 0; each lane owns a run of the member's tiles), then everybody's
    const int per_lane_tiles = (my_tiles + kWave - 1) / kWave;
    const int l0 = min(lane * per_lane_tiles, my_tiles), l1 = min(l0 + per_lane_tiles, my_tiles);
    double run = 0.0, incl = 0.0;
    if (wave == 0) {
        for (int t = l0; t < l1; ++t) run += tile_sum[t];
        incl = wave_inclusive_scan(run);
        if (lane == kWave - 1) sh_local_total = incl;
    }
    __syncthreads();
    const double local_total = sh_local_total;
    {
        unsigned mine = 0u;
        if (threadIdx.x == 0) mine = half_of(local_total, 0);
        if (threadIdx.x == 1) mine = half_of(local_total, 1);
        team_exchange(team, mine);
    }
    double total = 0.0, before = 0.0;
    for (int m = 0; m < team.size; ++m) {
        if (m == team.member) before = total;
        total += double_at(g_sh.words, m, 0);
    }
    const float u_draw = a.walk ? as_global(a.draw_uniforms)[bn] : as_global(a.uniforms)[static_cast<size_t>(b) * a.N];
    const double target = static_cast<double>(u_draw) * total;
    // the member whose run contains the target: the first whose running total exceeds it and that
    // has mass; rounding only: the last one that has mass
    int owner = -1, last_mass = 0;
    {
        double acc = 0.0;
        for (int m = 0; m < team.size; ++m) {
            const double tm = double_at(g_sh.words, m, 0);
            if (tm > 0.0) last_mass = m;
            if (owner < 0 && tm > 0.0 && acc + tm > target) owner = m;
            acc += tm;
        }
        if (owner < 0) owner = last_mass;
    }
    const bool mine_it = owner == team.member;
    const double local_target = target - before;

    // ---- the owner locates the tile that contains the target (wave 0) ...
    if (mine_it && wave == 0) {
        const unsigned long long hit = __ballot(incl > local_target && run > 0.0);
        int lane_owner = hit ? (__ffsll(static_cast<long long>(hit)) - 1) : -1;
        if (lane_owner < 0) {           // rounding only: last lane that has mass
            const unsigned long long any = __ballot(run > 0.0);
            lane_owner = any ? (63 - __clzll(static_cast<long long>(any))) : 0;
        }
        if (lane == lane_owner) {
            double acc = incl - run;
            int found = -1, last = l0;
            double bef = acc;
            for (int t = l0; t < l1; ++t) {
                const double ts = tile_sum[t];
                if (ts > 0.0) last = t;
                if (found < 0 && acc + ts > local_target && ts > 0.0) { found = t; bef = acc; }
                acc += ts;
            }
            if (found < 0) {       // rounding only: last tile of the run that has mass
                found = last;
                bef = incl - run;
                for (int t = l0; t < last; ++t) bef += tile_sum[t];
            }
            sh_tile = t_lo + found;
            sh_before = bef;
        }
    }
    __syncthreads();

    // ---- ... and the token inside that tile (wave 0)
    int tok = 0;
    if (mine_it && wave == 0) {
        const int t = sh_tile;
        const double rem = local_target - sh_before;       // mass to cover inside the tile
        float r[PER_LANE];
        rt_.load(t, lane, r);
        float ls = 0.f;
#pragma unroll
        for (int i = 0; i < PER_LANE; ++i) ls += r[i];
        const double lsd = static_cast<double>(ls);
        const double incl2 = wave_inclusive_scan(lsd);
        const unsigned long long hit = __ballot(incl2 > rem && ls > 0.f);
        int lane_owner = hit ? (__ffsll(static_cast<long long>(hit)) - 1) : -1;
        if (lane_owner < 0) {
            const unsigned long long any = __ballot(ls > 0.f);
            lane_owner = any ? (63 - __clzll(static_cast<long long>(any))) : 0;
        }
        if (lane == lane_owner) {
            double acc = incl2 - lsd;
            int found = -1, last = 0;
            double lo = acc, hi = acc;
            for (int i = 0; i < PER_LANE; ++i) {
                const double ri = static_cast<double>(r[i]);
                if (ri > 0.0) last = i;
                if (found < 0 && ri > 0.0 && acc + ri > rem) { found = i; lo = acc; hi = acc + ri; }
                acc += ri;
            }
            if (found < 0) { found = last; lo = rem; hi = rem; }
            int tk = t * TILE + lane * PER_LANE + found;
            if (tk >= V) tk = V - 1;
            as_global(a.bonus)[b] = tk;
            sh_tile = tk;                             // (the tile number is no longer needed)
            const double gap = fmin(fabs(rem - lo), fabs(hi - rem));
            if (gap < 1e-6 * total) atomicAdd(&a.counters[MPV_COUNTER_NEAR_TIE_BONUS], 1u);
        }
    }
    if (a.walk) {
        // Sec. 3.2: if the drawn token is a child's token the walk moves to that child (the
        // first such child in list order), otherwise it ends here.  Everybody needs the token.
        __syncthreads();
        {
            unsigned mine = 0u;
            if (threadIdx.x == 0 && mine_it) mine = static_cast<unsigned>(sh_tile);
            team_exchange(team, mine);
        }
        tok = static_cast<int>(g_sh.words[owner * kExchWords]);
        if (wave == 0) {
            const int k = tree.nchild[n];
            bool same = false;
            if (lane < k) same = as_global(a.tokens)[static_cast<size_t>(b) * a.N + tree.child_list[tree.child_off[n] + lane]] == tok;
            const unsigned long long m = __ballot(same);
            if (m) {
                const int to = tree.child_list[tree.child_off[n] + __ffsll(static_cast<long long>(m)) - 1];
                if (lane == 0) {
                    if (leader) st_relaxed(&ws.cur[b], to);
                    // Naive and SpecTr test children of an inner node before they draw there; NSS and leaves draw at once
                    sh_next = (a.walk >= 2 && tree.nchild[to] > 0) ? b * a.N + to : a.B * a.N + b;
                }
            } else if (leader) {
                if (lane == 0) write_path(tree, a, b, n);
                if (a.dbg_accept && lane < a.N)
                    as_global(a.dbg_accept)[static_cast<size_t>(b) * a.N + lane] =
                        lane == 0 ? 1.f : static_cast<float>(ld_shared_f64(&ws.atest[static_cast<size_t>(b) * a.N + lane]));
            }
        }
    }

    // ---- optional: the normalised distribution itself
    if (a.dbg_resid) {
        const double inv = 1.0 / total;
        float* out = a.dbg_resid + static_cast<size_t>(b) * V;
        for (int t = t_lo + wave; t < t_hi; t += NW) {
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
    int32_t* mb = static_cast<int32_t*>(take(kMaxTeams * 4));
    unsigned long long* kn = static_cast<unsigned long long*>(take(static_cast<size_t>(p->B) * 8));
    unsigned long long* ac = static_cast<unsigned long long*>(take(static_cast<size_t>(p->B) * 8));
    int32_t* de = static_cast<int32_t*>(take(static_cast<size_t>(p->B) * 4));
    int32_t* cu = static_cast<int32_t*>(take(static_cast<size_t>(p->B) * 4));
    TreeDesc* tr = static_cast<TreeDesc*>(take(sizeof(TreeDesc)));
    unsigned long long* ex = static_cast<unsigned long long*>(take(static_cast<size_t>(kMaxGrid) * 2 * kExchWords * 8));
    unsigned long long* tt = static_cast<unsigned long long*>(take(static_cast<size_t>(kMaxTeams) * 2 * 8));
    int32_t* ar = static_cast<int32_t*>(take(kMaxTeams * 4));
    Launch* la = static_cast<Launch*>(take(sizeof(Launch)));
    if (ws) { ws->exch = ex; ws->team_task = tt; ws->arrived = ar; ws->launch = la; }
    if (ws) { ws->At = At; ws->Ad = Ad; ws->cfin = cf; ws->aux = ax; ws->a0 = a0; ws->atest = at; ws->queue = qu; ws->qctl = qc; ws->mailbox = mb; ws->known = kn; ws->acc = ac; ws->decided = de; ws->cur = cu; ws->tree = tr; }
    return off < 256 ? 256 : off;
}

// Calls fn(b0, b1) for every run [b0, b1) of consecutive equal rows of rows[B][N], in order, until fn returns false.
template <typename F>
static void for_each_run(const int32_t* rows, int32_t B, int32_t N, F fn) {
    for (int32_t b0 = 0; b0 < B;) {
        int32_t b1 = b0 + 1;
        while (b1 < B && memcmp(rows + static_cast<size_t>(b0) * N, rows + static_cast<size_t>(b1) * N, sizeof(int32_t) * N) == 0)
            ++b1;
        if (!fn(b0, b1)) return;
        b0 = b1;
    }
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

// How a launch is shaped: G workgroups per team so that a member's part of a row fits on chip
// (kMaxTeam at most: beyond that the rest of a part is re-read in every sweep), as many teams
// as there can be tasks at once, three workgroups per compute unit at most.
struct Shape { int team_size, teams, part_vecs, same_xcd; };

// Workgroups of a task kernel that one compute unit holds at a time, as the runtime computes it
// from the kernel's registers and LDS (3 by design); a team never has more members than can be
// resident together.
template <class K>
static int resident_per_cu(K kernel) {
    int n = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, kernel, kTaskBlock, 0) != hipSuccess || n < 1) {
        (void)hipGetLastError();
        n = 1;
    }
    return n;
}

template <class E>
static Shape launch_shape(const mpv_problem* p, int tasks, int per_cu) {
    Shape s;
    const int nvec = (p->V + E::VEC - 1) / E::VEC;
    const int slots = per_cu * compute_units() < kMaxGrid ? per_cu * compute_units() : kMaxGrid;      // workgroups that can be resident
    // The fewest members whose kept parts (plus the one overflow slot a sweep hides) hold a row:
    // the most teams, which is what counts when there are more trees than teams.  With fewer
    // trees a task's own time counts: more members, parts of about 2048 vectors (measured: shorter
    // parts no longer pay for the larger exchange), as long as every tree still has a team.
    int g = 1;
    while (g < kMaxTeam && static_cast<long long>(g) * (kPartCapacity + kTaskBlock / 2) < nvec) ++g;
    while (g < kMaxTeam && slots / (g + 1) >= p->B && static_cast<long long>(g) * 2048 < nvec) ++g;
    int teams = slots / g;
    if (teams > kMaxTeams) teams = kMaxTeams;
    if (teams > tasks) teams = tasks;
    if (teams < 1) teams = 1;
    // workgroup i runs on chiplet i % 8: with a multiple of 8 teams every team can stay on one chiplet
    s.same_xcd = (g > 1 && teams >= 8) ? 1 : 0;
    if (s.same_xcd) teams -= teams % 8;
    s.team_size = g;
    s.teams = teams;
    const int tiles = (nvec + kWave - 1) / kWave;                 // wave tiles of 64 vectors
    s.part_vecs = ((tiles + g - 1) / g) * kWave;
    return s;
}

template <class E>
static int launch_all(const mpv_problem* p, const Plan& plan, const Workspace& ws, const Args& a, hipStream_t s) {
    TreeDesc tree = plan.tree;
    (void)hipGetLastError();    // a stale error left by the caller's own HIP calls is not ours
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
    static const int per_cu[3] = {resident_per_cu(node_task_kernel<E, MPV_METHOD_SPECINFER>),
                                  resident_per_cu(node_task_kernel<E, MPV_METHOD_TRAVERSAL>),
                                  resident_per_cu(node_task_kernel<E, kKindAcceptance>)};
    const Shape shape = launch_shape<E>(p, tasks, per_cu[a.estimate == 2 ? 2 : (p->method == MPV_METHOD_TRAVERSAL ? 1 : 0)]);
    q.teams = shape.teams;
    q.team_size = shape.team_size;
    q.part_vecs = shape.part_vecs;
    q.same_xcd = shape.same_xcd;
    q.split_node = -1;
    if (p->method == MPV_METHOD_TRAVERSAL && a.lazy && p->B >= q.teams) {
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
        const dim3 grid(static_cast<unsigned>(q.teams * q.team_size)), block(kTaskBlock);
        if (a.estimate == 2) {
            launch(MPV_KERNEL_NODE_TASK, node_task_kernel<E, kKindAcceptance>, grid, block, s, const_cast<const Launch*>(ws.launch));
        } else if (p->method != MPV_METHOD_TRAVERSAL) {      // NSS, Naive and SpecTr are variants of the top-down kernel
            launch(MPV_KERNEL_NODE_TASK, node_task_kernel<E, MPV_METHOD_SPECINFER>, grid, block, s, const_cast<const Launch*>(ws.launch));
        } else {
            launch(MPV_KERNEL_NODE_TASK, node_task_kernel<E, MPV_METHOD_TRAVERSAL>, grid, block, s, const_cast<const Launch*>(ws.launch));
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

// part_of_batch: the buffers are those of a larger batch moved on by a whole number of trees (the two
// logit pointers by the same number of bytes, so the rows of a pair still share their offset modulo 16
// bytes, which is what the kernels rely on; the caller has checked the batch's own pointers);
// keep_counters: add to the counters instead of starting them at zero.
// context_node: see Args (device pointer, already moved on to the run's first tree).
static int verify_with_workspace(const mpv_problem* problem, const mpv_buffers* buf, void* workspace,
                                 size_t workspace_bytes, void* hip_stream, bool part_of_batch = false,
                                 bool keep_counters = false, const int32_t* context_node = nullptr);

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
                                 size_t workspace_bytes, void* hip_stream, bool part_of_batch, bool keep_counters,
                                 const int32_t* context_node) {
    mpv::Plan plan;
    const int rc = mpv::validate(problem, &plan);
    if (rc != MPV_OK) return rc;
    if (!buf) return MPV_ERR_NULL;
    if (problem->B == 0) return MPV_OK;
    if (!buf->target_logits || !buf->draft_logits || !buf->tokens || !buf->uniforms || !buf->accept_len ||
        !buf->path_nodes || !buf->path_tokens || !buf->bonus_token || !buf->counters)
        return MPV_ERR_NULL;
    if (!part_of_batch &&
        ((reinterpret_cast<uintptr_t>(buf->target_logits) & 15u) || (reinterpret_cast<uintptr_t>(buf->draft_logits) & 15u)))
        return MPV_ERR_ALIGNMENT;
    if (((reinterpret_cast<uintptr_t>(buf->target_logits) ^ reinterpret_cast<uintptr_t>(buf->draft_logits)) & 15u) != 0)
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
    a.keep_counters = keep_counters ? 1 : 0;
    a.context_node = context_node;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (problem->logit_dtype == MPV_DTYPE_F32) return mpv::launch_all<mpv::ElemF32>(problem, plan, ws, a, s);
    return mpv::launch_all<mpv::ElemBF16>(problem, plan, ws, a, s);
}

int mpv_merge_duplicates(const int32_t* parent, const int32_t* tokens, int32_t B, int32_t N,
                         int32_t* merged_parent, int32_t* context_node) {
    if (!parent || !merged_parent || (B > 0 && !tokens)) return MPV_ERR_NULL;
    if (B < 0 || N < 1) return MPV_ERR_BAD_SHAPE;
    if (N > MPV_MAX_NODES) return MPV_ERR_UNSUPPORTED;
    if (parent[0] != -1) return MPV_ERR_BAD_TREE;
    for (int n = 1; n < N; ++n)
        if (parent[n] < 0 || parent[n] >= n) return MPV_ERR_BAD_TREE;
    for (int32_t b = 0; b < B; ++b) {
        const int32_t* tok = tokens + static_cast<size_t>(b) * N;
        int32_t* out = merged_parent + static_cast<size_t>(b) * N;
        // stands_for[n]: the node of slot n's context; entries[c]: the slots already placed under the
        // context node c that are nodes themselves (one per distinct token), in slot order
        int32_t stands_for[MPV_MAX_NODES];
        int8_t entries[MPV_MAX_NODES][MPV_MAX_NODES];
        int8_t count[MPV_MAX_NODES];
        memset(count, 0, sizeof(count));
        stands_for[0] = 0;
        out[0] = -1;
        for (int n = 1; n < N; ++n) {
            const int under = stands_for[parent[n]];
            out[n] = under;
            stands_for[n] = n;
            for (int j = 0; j < count[under]; ++j) {
                const int m = entries[under][j];
                if (tok[m] == tok[n]) { stands_for[n] = m; break; }
            }
            if (stands_for[n] == n) entries[under][count[under]++] = static_cast<int8_t>(n);
        }
        if (context_node) memcpy(context_node + static_cast<size_t>(b) * N, stands_for, sizeof(int32_t) * N);
    }
    return MPV_OK;
}

int mpv_verify_merged(const mpv_problem* problem, const int32_t* merged_parent, const int32_t* context_node,
                      const mpv_buffers* buf, void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!problem || !buf) return MPV_ERR_NULL;
    if (problem->B < 0 || problem->N < 1 || problem->V < 1) return MPV_ERR_BAD_SHAPE;
    if (problem->B == 0) return MPV_OK;
    if (!merged_parent) return MPV_ERR_NULL;
    if (problem->method == MPV_METHOD_SPECTR && !context_node) return MPV_ERR_NULL;
    if (problem->method != MPV_METHOD_SPECTR) context_node = nullptr;      // the other rules never accept a repeat
    const int32_t B = problem->B, N = problem->N;
    // first pass: every run of equal shapes is a valid problem, and the workspace holds the largest
    // (its size depends on the number of trees and of nodes only, and grows with both)
    mpv_problem run = *problem;
    int rc = MPV_OK;
    mpv::for_each_run(merged_parent, B, N, [&](int32_t b0, int32_t b1) {
        run.B = b1 - b0;
        run.parent = merged_parent + static_cast<size_t>(b0) * N;
        mpv::Plan plan;
        rc = mpv::validate(&run, &plan);
        return rc == MPV_OK;
    });
    if (rc != MPV_OK) return rc;
    run.B = B;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) || workspace_bytes < mpv::carve(&run, nullptr, nullptr))
        return MPV_ERR_WORKSPACE;
    if ((reinterpret_cast<uintptr_t>(buf->target_logits) & 15u) || (reinterpret_cast<uintptr_t>(buf->draft_logits) & 15u))
        return MPV_ERR_ALIGNMENT;
    const size_t elem = problem->logit_dtype == MPV_DTYPE_F32 ? 4 : 2;
    const size_t V = static_cast<size_t>(problem->V), D = static_cast<size_t>(problem->max_depth);
    auto moved = [](const void* p, size_t bytes) -> const void* { return p ? static_cast<const char*>(p) + bytes : nullptr; };
    auto moved_out = [](void* p, size_t bytes) -> void* { return p ? static_cast<char*>(p) + bytes : nullptr; };
    bool first = true;
    mpv::for_each_run(merged_parent, B, N, [&](int32_t b0, int32_t b1) {
        run.B = b1 - b0;
        run.parent = merged_parent + static_cast<size_t>(b0) * N;
        const size_t t = static_cast<size_t>(b0), tn = t * N;
        mpv_buffers part = *buf;
        part.target_logits = moved(buf->target_logits, tn * V * elem);
        part.draft_logits = moved(buf->draft_logits, tn * V * elem);
        part.tokens = static_cast<const int32_t*>(moved(buf->tokens, tn * 4));
        part.uniforms = static_cast<const float*>(moved(buf->uniforms, tn * 4));
        part.draw_uniforms = static_cast<const float*>(moved(buf->draw_uniforms, tn * 4));
        part.accept_len = static_cast<int32_t*>(moved_out(buf->accept_len, t * 4));
        part.path_nodes = static_cast<int32_t*>(moved_out(buf->path_nodes, t * D * 4));
        part.path_tokens = static_cast<int32_t*>(moved_out(buf->path_tokens, t * D * 4));
        part.bonus_token = static_cast<int32_t*>(moved_out(buf->bonus_token, t * 4));
        part.stats = static_cast<float*>(moved_out(buf->stats, tn * 4 * 4));
        part.edge_probs = static_cast<float*>(moved_out(buf->edge_probs, tn * 2 * 4));
        part.accept_prob = static_cast<float*>(moved_out(buf->accept_prob, tn * 4));
        part.final_residual = static_cast<float*>(moved_out(buf->final_residual, t * V * 4));
        rc = verify_with_workspace(&run, &part, workspace, workspace_bytes, hip_stream, true, !first,
                                   context_node ? context_node + tn : nullptr);
        first = false;
        return rc == MPV_OK;
    });
    return rc;
}

// part_of_batch, keep_counters: as for verify_with_workspace
static int block_efficiency_with_workspace(const mpv_problem* problem, const void* target_logits, const void* draft_logits,
                                           const int32_t* tokens, void* workspace, size_t workspace_bytes,
                                           float* reach_prob, float* expected, uint32_t* counters, void* hip_stream,
                                           bool part_of_batch, bool keep_counters, const int32_t* context_node = nullptr) {
    mpv::Plan plan;
    const int rc = mpv::validate(problem, &plan);
    if (rc != MPV_OK) return rc;
    if (problem->B == 0) return MPV_OK;
    if (!target_logits || !draft_logits || !tokens || !expected || !counters) return MPV_ERR_NULL;
    if (!part_of_batch && ((reinterpret_cast<uintptr_t>(target_logits) & 15u) || (reinterpret_cast<uintptr_t>(draft_logits) & 15u)))
        return MPV_ERR_ALIGNMENT;
    if (((reinterpret_cast<uintptr_t>(target_logits) ^ reinterpret_cast<uintptr_t>(draft_logits)) & 15u) != 0)
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
    a.keep_counters = keep_counters ? 1 : 0;
    a.context_node = context_node;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (problem->logit_dtype == MPV_DTYPE_F32) return mpv::launch_all<mpv::ElemF32>(problem, plan, ws, a, s);
    return mpv::launch_all<mpv::ElemBF16>(problem, plan, ws, a, s);
}

int mpv_block_efficiency(const mpv_problem* problem, const void* target_logits, const void* draft_logits,
                         const int32_t* tokens, void* workspace, size_t workspace_bytes,
                         float* reach_prob, float* expected, uint32_t* counters, void* hip_stream) {
    return block_efficiency_with_workspace(problem, target_logits, draft_logits, tokens, workspace, workspace_bytes,
                                           reach_prob, expected, counters, hip_stream, false, false);
}

int mpv_block_efficiency_merged(const mpv_problem* problem, const int32_t* merged_parent, const int32_t* context_node,
                                const void* target_logits, const void* draft_logits, const int32_t* tokens, void* workspace,
                                size_t workspace_bytes, float* reach_prob, float* expected, uint32_t* counters,
                                void* hip_stream) {
    if (!problem) return MPV_ERR_NULL;
    if (problem->B < 0 || problem->N < 1 || problem->V < 1) return MPV_ERR_BAD_SHAPE;
    if (problem->B == 0) return MPV_OK;
    if (!merged_parent) return MPV_ERR_NULL;
    if (problem->method == MPV_METHOD_SPECTR && !context_node) return MPV_ERR_NULL;
    if (problem->method != MPV_METHOD_SPECTR) context_node = nullptr;
    mpv_problem run = *problem;
    int rc = MPV_OK;
    mpv::for_each_run(merged_parent, problem->B, problem->N, [&](int32_t b0, int32_t b1) {
        run.B = b1 - b0;
        run.parent = merged_parent + static_cast<size_t>(b0) * problem->N;
        mpv::Plan plan;
        rc = mpv::validate(&run, &plan);
        return rc == MPV_OK;
    });
    if (rc != MPV_OK) return rc;
    run.B = problem->B;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) || workspace_bytes < mpv::carve(&run, nullptr, nullptr))
        return MPV_ERR_WORKSPACE;
    if (!target_logits || !draft_logits || !tokens || !expected || !counters) return MPV_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(target_logits) & 15u) || (reinterpret_cast<uintptr_t>(draft_logits) & 15u))
        return MPV_ERR_ALIGNMENT;
    const size_t elem = problem->logit_dtype == MPV_DTYPE_F32 ? 4 : 2;
    const size_t N = static_cast<size_t>(problem->N), V = static_cast<size_t>(problem->V);
    bool first = true;
    mpv::for_each_run(merged_parent, problem->B, problem->N, [&](int32_t b0, int32_t b1) {
        run.B = b1 - b0;
        run.parent = merged_parent + static_cast<size_t>(b0) * N;
        const size_t t = static_cast<size_t>(b0), tn = t * N;
        rc = block_efficiency_with_workspace(&run, static_cast<const char*>(target_logits) + tn * V * elem,
                                             static_cast<const char*>(draft_logits) + tn * V * elem, tokens + tn,
                                             workspace, workspace_bytes, reach_prob ? reach_prob + tn : nullptr,
                                             expected + t, counters, hip_stream, true, !first,
                                             context_node ? context_node + tn : nullptr);
        first = false;
        return rc == MPV_OK;
    });
    return rc;
}


// part_of_batch, keep_counters: as for verify_with_workspace
static int acceptance_rates_with_workspace(const mpv_problem* problem, const void* target_logits, const void* draft_logits,
                                           void* workspace, size_t workspace_bytes, float* alpha, uint32_t* counters,
                                           void* hip_stream, bool part_of_batch, bool keep_counters) {
    mpv::Plan plan;
    const int rc = mpv::validate(problem, &plan);
    if (rc != MPV_OK) return rc;
    if (problem->method == MPV_METHOD_TRAVERSAL) return MPV_ERR_UNSUPPORTED;     // not an OTLP solver: App. C has no rate for it
    if (problem->B == 0) return MPV_OK;
    if (!target_logits || !draft_logits || !alpha || !counters) return MPV_ERR_NULL;
    if (!part_of_batch && ((reinterpret_cast<uintptr_t>(target_logits) & 15u) || (reinterpret_cast<uintptr_t>(draft_logits) & 15u)))
        return MPV_ERR_ALIGNMENT;
    if (((reinterpret_cast<uintptr_t>(target_logits) ^ reinterpret_cast<uintptr_t>(draft_logits)) & 15u) != 0)
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
    a.keep_counters = keep_counters ? 1 : 0;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (problem->logit_dtype == MPV_DTYPE_F32) return mpv::launch_all<mpv::ElemF32>(problem, plan, ws, a, s);
    return mpv::launch_all<mpv::ElemBF16>(problem, plan, ws, a, s);
}

int mpv_acceptance_rates(const mpv_problem* problem, const void* target_logits, const void* draft_logits,
                         void* workspace, size_t workspace_bytes, float* alpha, uint32_t* counters, void* hip_stream) {
    return acceptance_rates_with_workspace(problem, target_logits, draft_logits, workspace, workspace_bytes, alpha, counters,
                                           hip_stream, false, false);
}

int mpv_acceptance_rates_merged(const mpv_problem* problem, const int32_t* merged_parent, const void* target_logits,
                                const void* draft_logits, void* workspace, size_t workspace_bytes, float* alpha,
                                uint32_t* counters, void* hip_stream) {
    if (!problem) return MPV_ERR_NULL;
    if (problem->B < 0 || problem->N < 1 || problem->V < 1) return MPV_ERR_BAD_SHAPE;
    if (problem->method == MPV_METHOD_TRAVERSAL) return MPV_ERR_UNSUPPORTED;
    if (problem->B == 0) return MPV_OK;
    if (!merged_parent) return MPV_ERR_NULL;
    mpv_problem run = *problem;
    int rc = MPV_OK;
    mpv::for_each_run(merged_parent, problem->B, problem->N, [&](int32_t b0, int32_t b1) {
        run.B = b1 - b0;
        run.parent = merged_parent + static_cast<size_t>(b0) * problem->N;
        mpv::Plan plan;
        rc = mpv::validate(&run, &plan);
        return rc == MPV_OK;
    });
    if (rc != MPV_OK) return rc;
    run.B = problem->B;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) || workspace_bytes < mpv::carve(&run, nullptr, nullptr))
        return MPV_ERR_WORKSPACE;
    if (!target_logits || !draft_logits || !alpha || !counters) return MPV_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(target_logits) & 15u) || (reinterpret_cast<uintptr_t>(draft_logits) & 15u))
        return MPV_ERR_ALIGNMENT;
    const size_t elem = problem->logit_dtype == MPV_DTYPE_F32 ? 4 : 2;
    const size_t N = static_cast<size_t>(problem->N), V = static_cast<size_t>(problem->V);
    bool first = true;
    mpv::for_each_run(merged_parent, problem->B, problem->N, [&](int32_t b0, int32_t b1) {
        run.B = b1 - b0;
        run.parent = merged_parent + static_cast<size_t>(b0) * N;
        const size_t tn = static_cast<size_t>(b0) * N;
        rc = acceptance_rates_with_workspace(&run, static_cast<const char*>(target_logits) + tn * V * elem,
                                             static_cast<const char*>(draft_logits) + tn * V * elem, workspace,
                                             workspace_bytes, alpha + tn, counters, hip_stream, true, !first);
        first = false;
        return rc == MPV_OK;
    });
    return rc;
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
