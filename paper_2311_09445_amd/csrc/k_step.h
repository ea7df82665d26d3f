// One iteration of Listing 2 whose update targets the batch it draws: sampling and update as one kernel, rows and weights in a second.
// Part of per_kernels.hip (included inside namespace per, in the order given there); not a stand-alone header.

// ---------------------------------------------------------------------------------
// the whole step, one workgroup per subtree
// ---------------------------------------------------------------------------------
// Stratified targets grow with the sample number and the walk is monotone in the target, so the samples
// that end under one node of the tree are a contiguous run of sample numbers.  Workgroup b of tree t owns
// the subtree under node b of height ho ("owner height").  It finds its run of samples, walks them down
// (the way from the root to node b is the same for all of them, so it is tabulated once; the heights
// 1 .. ho-1 of its own subtree come from an LDS copy, the leaf groups from memory), and
// then applies the update of exactly those samples to its own subtree: every leaf, every height-1 node and
// every higher node of the subtree is read and written by this workgroup only, so the update needs no claim
// phase, no atomics and no second pass over the leaf groups (they are still in LDS from the walk).
// Sampling sees the tree as it was before the call because a workgroup finishes all its walks before it
// changes anything, and what all workgroups read is not written by this kernel at all: the way from the
// root to every owner's node (the left and right block sums of each binary step, in the walk's own
// arithmetic), the mass in front of the node and the tree's total sit in a table built from the nodes
// of height ho and above by the kernel that ends the call before (k_step_epilogue), or by a small
// kernel in front when another call has changed the tree since (k_step_tables).  The new value of node b
// goes to a side array; the epilogue moves the side array into the level array, recomputes the heights
// above (so nothing is left stale), builds the tables of the next call, and turns the sampled values
// into importance weights (they are relative to the batch minimum, which is known only when every owner
// is done: the owners leave their values and, in slots, their minima).  The slots and the builders'
// counters alternate between two sets by the number of finished calls, which is counted on the device:
// every owner adds one to a counter when it is done (spread over kStepGroups counters, because atomics on
// one address queue up), and a workgroup that reads its own group's counter when it starts gets the
// number of finished calls whatever the others have already added.  (Owners that wait for each other
// inside the kernel to finish the weights themselves were tried: 512 workgroups polling the counters
// slowed the very atomics they waited for, + 9 us.  The whole call inside this kernel, with a wait built as a tree of
// counters and no memory fences, is there as an option (TAIL, tuning "step_tail"): 25.4 against 22.0 us per step
// on the 65536-sample workload; between the last owner's last store and the moment every workgroup knows that
// all have arrived lie 7 us, although that wait alone, with nothing else going on, takes 2 us.)
//
// Last writer: element j of the update targets the leaf drawn by sample pos[j] (no map: by sample j).  The
// samples of one leaf are neighbours in a workgroup's run, so the winner of a leaf is the largest j among
// the elements aimed at that run of samples.  With a map, builder workgroups in front of the grid first
// record for every sample the largest j aimed at it (an atomic max into a scratch word per sample that the
// sample's lane takes back out with an exchange); the owners wait for them at the point where they need the
// words, which the builders, being dispatched first and waiting for nothing, always reach.
constexpr int kStepTop = 4;          // most heights ho .. H-1
constexpr int kStepSub = 4;          // most heights 1 .. ho-1
constexpr uint32_t kStepPad = 4;     // sample numbers looked at in front of the estimated start of the run
constexpr uint32_t kNoKey = 0xFFFFFFFFu;
constexpr uint32_t kStepSpinLimit = 1u << 20;   // polls of a counter before a workgroup gives up
constexpr int kStepPathMax = kStepTop * 6;      // binary steps from the root to a node of the owner height

// What an owner needs of the tree above it (one entry per owner, rebuilt whenever the heights ho .. H change).
struct StepTable {
  float2 path[kStepPathMax];   // per binary step from the root to the node: (sum of the left block, flags); bit 0 of the flags:
                               // the node lies to the right; bit 1: the right block is not zero
  double mass;                 // sum of the nodes of height ho in front of it, as a fraction of the total (0 when that is 0)
  float total;                 // the root
  float node;                  // its own value
};

struct StepShape {
  float* top_ptr[kStepTop];        // height ho + i of tree 0 (i = 0: the level array of height ho)
  uint32_t top_stride[kStepTop];   // floats between trees
  uint32_t top_cnt[kStepTop];      // floats kept in LDS: whole child groups, n[ho+i+1] * K
  uint32_t top_n[kStepTop];        // real nodes n[ho+i]
  uint32_t top_off[kStepTop];      // where in LDS (floats)
  float* sub_ptr[kStepSub];        // height 1 + i of tree 0
  uint32_t sub_stride[kStepSub];
  uint32_t sub_cnt[kStepSub];      // nodes of that height under one owner: K^(ho-1-i)
  uint32_t sub_pad[kStepSub];      // nodes of that height in memory, padded to whole groups
  uint32_t sub_off[kStepSub];      // where in LDS (floats)
  uint32_t n_top, n_sub;           // H - ho, ho - 1
  uint32_t path_off;               // LDS: this owner's table entries (kStepPathMax float2)
  uint32_t rows_off;               // LDS: (block + 1) staging rows of K + 4 floats (16-byte aligned)
  uint32_t key_off;                // LDS: key[block + 2], wpos[block + 1], wval[block + 1], touch[block + 1]
  uint32_t owners;                 // n[ho]: owner workgroups per tree
  uint32_t builders;               // builder workgroups per tree in front of them (0: no position map)
  float* root;                     // root of tree 0
  uint32_t root_stride;
  float* side;                     // [T][side_stride] where the owners leave the new values of their nodes of height ho
  StepTable* tab;                  // [T][owners]
  uint32_t side_stride;
  unsigned long long* cnt;         // [T][kStepGroups] finished owners of group i, over all calls
  uint32_t* done;                  // [T][2][kStepDoneSlots] finished builders of this call (by parity of the call number)
  uint32_t* vmin;                  // [T][2][kVminSlots] smallest sampled values of this call (fp32 bits; by parity)
  uint32_t* inv;                   // [T][inv_stride] per sample: 1 + the largest update element aimed at it (zero between calls)
  uint32_t inv_stride;
  // when the call ends inside k_step (TAIL)
  uint32_t helpers;                // workgroups in front of the owners: builders and / or the builders of the next call's tables
  uint32_t table_blocks;           // how many of them build tables once every owner has arrived
  unsigned long long* cnt2;        // [T] groups of owners that have all arrived, over all such calls
  uint32_t* rel;                   // [T] number of finished calls: written when the last owner of a call has arrived (or by the epilogue)
};
struct StepTail { FieldTable ft; };   // rows of the sampled indices (io all null: none)
struct NoTail { uint32_t none; };
template <bool TAIL> using TailParam = typename std::conditional<TAIL, StepTail, NoTail>::type;
template <int LOGK, bool COHERENT>
__device__ __forceinline__ void build_tables(const StepShape& sh, uint32_t t, const float* src, bool from_side, uint32_t first,
                                             uint32_t count, float* top, float* skipped);
constexpr uint32_t kTableOwners = 8;   // owners whose tables one workgroup builds

__device__ __forceinline__ uint32_t owners_of_group(uint32_t owners, uint32_t i) {
  return i < owners ? (owners - i + kStepGroups - 1u) / kStepGroups : 0u;
}
__device__ __forceinline__ unsigned long long load_counter(const unsigned long long* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Balanced pairwise sum of the 2^m floats at p (half a child group at most: m < LOGK), in the order of group_sum and
// of the walk inside a group.
template <int LOGK>
__device__ __forceinline__ float block_sum(const float* p, uint32_t m) {
  if (m == 0) return p[0];
  if (m == 1) return p[0] + p[1];
  constexpr int MAXC = (1 << LOGK) / 8 > 1 ? (1 << LOGK) / 8 : 1;   // most chunks of four in half a group
  const uint32_t nc = 1u << (m - 2);
  float s[MAXC];
#pragma unroll
  for (int c = 0; c < MAXC; ++c) {
    const float4 x = *reinterpret_cast<const float4*>(p + 4 * ((uint32_t)c < nc ? c : 0));
    s[c] = (x.x + x.y) + (x.z + x.w);
  }
#pragma unroll
  for (int w = MAXC; w > 1; w >>= 1) {
    if ((uint32_t)w <= nc) {
#pragma unroll
      for (int c = 0; c < w / 2; ++c) s[c] = s[2 * c] + s[2 * c + 1];
    }
  }
  return s[0];
}

// Pairwise sum of the K floats of a staged row, in the order of group_sum.
template <int LOGK>
__device__ __forceinline__ float row_sum(const float* row) {
  if constexpr (LOGK == 1) {
    return row[0] + row[1];
  } else {
    constexpr int C = (1 << LOGK) / 4;
    const float4* r4 = reinterpret_cast<const float4*>(row);
    float s[C];
#pragma unroll
    for (int c = 0; c < C; ++c) {
      const float4 x = r4[c];
      s[c] = (x.x + x.y) + (x.z + x.w);
    }
#pragma unroll
    for (int w = C; w > 1; w >>= 1)
#pragma unroll
      for (int c = 0; c < w / 2; ++c) s[c] = s[2 * c] + s[2 * c + 1];
    return s[0];
  }
}

// The update of one chunk of a workgroup's samples, on LDS arrays indexed by slot: slot 0 carries what the
// chunk before left open, slot 1 + i belongs to lane i.
//   key[slot]   leaf of the slot's sample (kNoKey: none); key[block + 1] is always kNoKey
//   wpos[slot]  1 + the largest update element aimed at that sample (0: none), wval[slot] its value
//   rows[slot]  the K leaves of the sample's group as staged for the walk (K + 4 floats apart)
//   touch[slot] (group heads only) a leaf of the group was rewritten
// A run of equal keys is one leaf; its last writer is the largest wpos in the run.  A run of keys with equal
// key >> LOGK is one child group; the row of its first slot (the head) collects the new leaf values, and at
// the end of the run its pairwise sum is the new height-1 node.  When the chunk is not the workgroup's
// last, the runs that reach its last slot stay open and move to slot 0 of the next chunk.
// Three phases, a workgroup barrier after each; thread i works on slot i, thread 0 also on slot `block`.
struct ChunkLds {
  uint32_t* key;
  uint32_t* wpos;
  float* wval;
  uint32_t* touch;
  float* rows;
};
template <int LOGK>
__device__ __forceinline__ uint32_t group_head(const ChunkLds& c, uint32_t slot) {
  const uint32_t g = c.key[slot] >> LOGK;
  uint32_t h = slot;
  while (h > 0 && c.key[h - 1] != kNoKey && (c.key[h - 1] >> LOGK) == g) --h;
  return h;
}
// Phase A: the slot that ends a leaf's run hands the winner's value to the group head's row and to memory.
template <int LOGK>
__device__ __forceinline__ void chunk_leaves(const ChunkLds& c, uint32_t slot, uint32_t block, bool last_chunk,
                                             float* __restrict__ leaves, uint32_t& open_pos, float& open_val) {
  constexpr int K = 1 << LOGK;
  constexpr int ROW = K + 4;
  const uint32_t k = c.key[slot];
  if (k == kNoKey) return;
  const bool open = slot == block && !last_chunk;
  if (!open && c.key[slot + 1] == k) return;   // the run goes on
  uint32_t best = c.wpos[slot];
  float bv = c.wval[slot];
  uint32_t j = slot;
  while (j > 0 && c.key[j - 1] == k) {
    --j;
    if (c.wpos[j] > best) {
      best = c.wpos[j];
      bv = c.wval[j];
    }
  }
  if (open) {
    open_pos = best;
    open_val = bv;
    return;
  }
  if (best) {
    const uint32_t h = group_head<LOGK>(c, j);
    c.rows[(size_t)h * ROW + (k & (uint32_t)(K - 1))] = bv;
    c.touch[h] = 1u;
    __builtin_nontemporal_store(bv, leaves + k);   // (leaves the cache while the kernel goes on, not when it ends)
  }
}
// Phase B: the slot that ends a group's run recomputes the height-1 node from the head's row.  Returns the head
// of the run that stays open (only for slot == block of a chunk that is not the last), else kNoKey.
template <int LOGK>
__device__ __forceinline__ uint32_t chunk_groups(const ChunkLds& c, uint32_t slot, uint32_t block, bool last_chunk,
                                                 float* __restrict__ lvl1, float* sub1, uint32_t lo1) {
  constexpr int K = 1 << LOGK;
  constexpr int ROW = K + 4;
  const uint32_t k = c.key[slot];
  if (k == kNoKey) return kNoKey;
  const uint32_t g = k >> LOGK;
  const bool open = slot == block && !last_chunk;
  if (!open && c.key[slot + 1] != kNoKey && (c.key[slot + 1] >> LOGK) == g) return kNoKey;   // the run goes on
  const uint32_t h = group_head<LOGK>(c, slot);
  if (open) return h;
  if (c.touch[h]) {
    const float sum = row_sum<LOGK>(c.rows + (size_t)h * ROW);
    __builtin_nontemporal_store(sum, lvl1 + g);
    sub1[g - lo1] = sum;
  }
  return kNoKey;
}


// TAIL: the call ends inside this kernel.  An owner that is done with its update announces it (its group's counter; the
// last of a group goes on to a counter of groups; the last of all writes the call's number into a word everybody
// polls), moves the rows of its own samples while the others arrive, and once all have, turns its samples' values
// into weights; the helper workgroups in front of the grid wait for the same word and then do what the epilogue
// kernel does otherwise (height ho from the side array, the heights above, the next call's tables).  Nothing of
// this uses memory fences between workgroups, which on this GPU (several dies, each with its own second-level
// cache) cost several microseconds each: the few words that travel between workgroups (the owners' new nodes, the
// smallest sampled values, the counters) are written and read with device-scope atomic accesses, which go past
// the caches, and a workgroup announces itself only after they have completed.  All waits are bounded; the host
// launches this form only when all workgroups of the grid fit the GPU at once (a waiting workgroup holds its place).
// The tables of one buffer per GPU (the first with a single tree that asks) sit in this array instead of its arena:
// a kernel knows the array's address without its arguments, so an owner of k_step<.., .., true> fetches its entry
// while the arguments are still on their way, and the trip that needs both (the window of samples) starts a trip
// earlier.  That form has a fixed number of workgroups in front of the owners (kStepFront; those that are no
// builders return at once), because the owner's number must not depend on an argument either.
// (The host never names the array: a variable that host code refers to is reached through an address table in
// memory, one more trip; its address is reported by a kernel instead.)
static __device__ __align__(256) StepTable g_step_tab_static[kStepMaxOwners];
constexpr uint32_t kStepFront = 64;
constexpr uint32_t kStepEpilogueArgLines = (1u << 0) | (3u << 12) | (0x1FFu << 17);
constexpr uint32_t kStepOwnerArgLines = (1u << 0) | (1u << 2) | (1u << 4) | (1u << 12) | (0x7Fu << 15);   // 64-byte lines of the kernel arguments
__global__ void k_step_static_address(void** out) { *out = g_step_tab_static; }
// Who holds the array on each GPU.  A buffer that held it before may still have work in flight that reads or writes
// it, so a GPU whose array changes hands is drained first.
namespace {
struct StaticTables {
  std::mutex mu;
  const void* holder[kMaxDevices] = {};
  bool used[kMaxDevices] = {};
  void* addr[kMaxDevices] = {};
};
StaticTables& static_tables() {
  static StaticTables st;
  return st;
}
}  // namespace
// Gives `holder` the array of `device` (which must be the current one) if nobody holds it: its address, else null.
// `s`: a stream of the caller's that is not being captured (the address is asked for on it, once per GPU).
void* step_static_claim(const void* holder, int device, hipStream_t s) {
  if (device < 0 || device >= kMaxDevices) return nullptr;
  int current = -1;
  if (hipGetDevice(&current) != hipSuccess || current != device) return nullptr;
  StaticTables& st = static_tables();
  std::lock_guard<std::mutex> lock(st.mu);
  if (st.holder[device]) return st.holder[device] == holder ? st.addr[device] : nullptr;
  if (!st.addr[device]) {   // asked once per GPU: a kernel writes the address into pinned host memory
    void** slot = nullptr;
    if (hipHostMalloc(reinterpret_cast<void**>(&slot), sizeof(void*), hipHostMallocDefault) != hipSuccess) return nullptr;
    *slot = nullptr;
    hipLaunchKernelGGL(k_step_static_address, dim3(1), dim3(1), 0, s, slot);
    const bool ok = hipGetLastError() == hipSuccess && hipStreamSynchronize(s) == hipSuccess;
    void* got = ok ? *slot : nullptr;
    (void)hipHostFree(slot);
    if (!got) return nullptr;
    st.addr[device] = got;
  }
  if (st.used[device] && hipDeviceSynchronize() != hipSuccess) return nullptr;
  st.holder[device] = holder;
  st.used[device] = true;
  return st.addr[device];
}
void step_static_release(const void* holder, int device) {
  if (device < 0 || device >= kMaxDevices) return;
  StaticTables& st = static_tables();
  std::lock_guard<std::mutex> lock(st.mu);
  if (st.holder[device] == holder) st.holder[device] = nullptr;
}

template <int LOGK, bool TAIL, bool STATIC = false>
__global__ void __launch_bounds__(512)
k_step(Geom g, StepShape sh, uint32_t B, uint32_t size, float beta, uint32_t weight_mode, const float* __restrict__ u,
       RngArgs rng, uint32_t* out_idx, float* __restrict__ out_prio, float* out_w,
       const float* __restrict__ upd_prio, const uint32_t* __restrict__ upd_pos, TailParam<TAIL> tail) {
  constexpr int K = Fan<LOGK>::K;
  constexpr int LPS = Fan<LOGK>::LPS;
  constexpr int ROW = K + 4;
  static_assert(LOGK >= 3, "the staged walk needs K >= 8");
  static_assert(!(TAIL && STATIC), "the form that ends inside the kernel has its own helpers in front");
  // STATIC: this owner's table entry, asked for before anything that needs an argument (one tree only)
  [[maybe_unused]] float pre_total = 0.0f;
  [[maybe_unused]] double pre_mass = 0.0;
  [[maybe_unused]] float2 pre_path = make_float2(0.0f, 0.0f);
  if constexpr (STATIC) {
    uint32_t zero;
    asm volatile("v_mov_b32 %0, 0" : "=v"(zero));   // (a lane offset the compiler cannot see through: vector loads, issued here)
    const StepTable* early = g_step_tab_static + (blockIdx.x >= kStepFront ? blockIdx.x - kStepFront : 0u) + zero;
    pre_total = early->total;
    pre_mass = early->mass;
    // (lane i of every wave: step i of the way; no branch: every lane loads)
    pre_path = early->path[(threadIdx.x & 63u) < (uint32_t)kStepPathMax ? (threadIdx.x & 63u) : (uint32_t)kStepPathMax - 1u];
    asm volatile("" ::: "memory");   // (the loads stay in front of this line, and so in front of everything that waits for an argument)
  }
  constexpr int kArgLines = kernarg_lines<Geom, StepShape, uint32_t, uint32_t, float, uint32_t, const float*, RngArgs, uint32_t*,
                                         float*, float*, const float*, const uint32_t*>();
  // (STATIC: only the lines an owner reads: the first words of the geometry, the strides and pointers of heights 0
  // and 1, the scalars' pointers, and everything from the subtree's description on; a line costs 35 to 60 ns even in a
  // batch, and the builders, which read more, are not what the kernel waits for)
  if constexpr (STATIC) touch_kernel_argument_lines<kStepOwnerArgLines>();
  else touch_kernel_arguments<kArgLines>();
  extern __shared__ __attribute__((aligned(16))) float lds[];
  __shared__ uint32_t s_u32[8];
  const uint32_t t = blockIdx.y;
  const uint32_t tid = threadIdx.x;
  const uint32_t BD = blockDim.x;
  const unsigned lane = tid & 63u;
  const unsigned wave = tid >> 6;
  const unsigned long long* cnt = sh.cnt + (size_t)t * kStepGroups;
  uint32_t* inv = sh.inv + (size_t)t * sh.inv_stride;
  const int n_top = (int)sh.n_top, n_sub = (int)sh.n_sub;
  const uint32_t n_steps = (uint32_t)n_top * LOGK;
  float* side_ho = sh.side + (size_t)t * sh.side_stride;
  const StepTable* tab = sh.tab + (size_t)t * sh.owners;

  // Waits (bounded) until the call's number `target` stands in the word that the last owner to arrive writes.
  auto wait_release = [&](uint32_t target) -> bool {
    if (wave == 0) {
      uint32_t spins = 0, ok = 1;
      for (;;) {
        uint32_t v = lane == 0 ? __hip_atomic_load(sh.rel + t, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0u;
        v = (uint32_t)__shfl((int)v, 0);
        if ((int32_t)(v - target) >= 0) break;
        if (++spins > kStepSpinLimit) {
          ok = 0;
          break;
        }
        __builtin_amdgcn_s_sleep(2);
      }
      if (lane == 0) {
        s_u32[0] = ok;
        if (!ok) atomicOr(&g.status[t], 8u);
      }
    }
    __syncthreads();
    const bool ok = s_u32[0] != 0;
    __syncthreads();
    return ok;
  };

  // ------------------------------------------------------------------ helper workgroups: builders (position map only), table builders (TAIL)
  const uint32_t front = STATIC ? kStepFront : (TAIL ? sh.helpers : sh.builders);   // workgroups in front of the owners
  if (blockIdx.x < front) {
    if (STATIC && blockIdx.x >= sh.builders) return;   // (there to keep the owners' numbers fixed)
    // The number of finished calls.  Without TAIL: the owners of this call cannot finish before every builder has, so
    // the count of group 0 is still that of the calls before.  With TAIL the owners' counters may already have moved
    // when a helper starts late, so the word that ends a call is read instead: it cannot move before every helper
    // has said (below) that it has read it.
    unsigned long long calls;
    if constexpr (TAIL) calls = __hip_atomic_load(sh.rel + t, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else calls = load_counter(cnt) / owners_of_group(sh.owners, 0);
    const uint32_t par = (uint32_t)calls & 1u;
    const uint32_t max_seen = read_max_bits(g, t);
    uint32_t mx = 0, f_idx = 0, f_prio = 0, acc = 0;
    for (uint32_t j = blockIdx.x * BD + tid; blockIdx.x < sh.builders && j < B; j += sh.builders * BD) {
      const uint32_t at = upd_pos[(size_t)t * B + j];
      const float v = upd_prio[(size_t)t * B + j];
      if (!(at < B)) f_idx = 1u;
      else if (!valid_priority(v)) f_prio = 2u;
      else {
        acc |= atomicMax(&inv[at], j + 1u);   // (returning: its arrival says that it has been performed)
        const uint32_t vb = v > 0.0f ? __float_as_uint(v) : 0u;
        mx = vb > mx ? vb : mx;
      }
    }
    // nothing can be sampled (and no element is valid) when the tree's total is not positive
    if (blockIdx.x < sh.builders) {
      const bool positive = tab[0].total > 0.0f;
      if (positive) {
        raise_max(g, t, mx, max_seen);
        if (f_idx | f_prio) atomicOr(&g.status[t], f_idx | f_prio);
      } else if (B) {
        if (tid == 0) atomicOr(&g.status[t], 1u);
      }
    }
    asm volatile("" ::"v"(acc));
    __syncthreads();   // every lane's atomics have returned
    if (tid == 0) atomicAdd(sh.done + ((size_t)t * 2 + par) * kStepDoneSlots + blockIdx.x % kStepDoneSlots, 1u);
    if constexpr (TAIL) {
      if (blockIdx.x < sh.table_blocks && wait_release((uint32_t)calls + 1u)) {
        __shared__ float skipped[kTableOwners * kStepPathMax];
        const uint32_t first = blockIdx.x * kTableOwners;
        const uint32_t count = sh.owners - first < kTableOwners ? sh.owners - first : kTableOwners;
        build_tables<LOGK, true>(sh, t, side_ho, true, first, count, lds, skipped);
      }
    }
    return;
  }

  // ------------------------------------------------------------------ owner workgroup b
  const uint32_t b = blockIdx.x - front;
  const uint32_t my_group = b % kStepGroups;
  float* sub = lds;                                   // heights 1 .. ho-1 of the own subtree, at sub_off[i]
  // per binary step from the root to b: the sum of the left block; bit 0: b lies to the right, bit 1: the right block is not zero
  float2* path = reinterpret_cast<float2*>(lds + sh.path_off);
  ChunkLds c;
  c.rows = lds + sh.rows_off;
  c.key = reinterpret_cast<uint32_t*>(lds + sh.key_off);
  c.wpos = c.key + (BD + 2);
  c.wval = reinterpret_cast<float*>(c.wpos + (BD + 1));
  c.touch = reinterpret_cast<uint32_t*>(c.wval + (BD + 1));

  bool tail_has_rows = false;
  if constexpr (TAIL)
    for (uint32_t f = 0; f < tail.ft.n_fields; ++f) tail_has_rows = tail_has_rows || tail.ft.io[f] != nullptr;
  PER_TRACE_DECL;
  PER_MARK(0);
  // ---- trip 1: the number of finished calls, this owner's table, the own subtree's heights, the running maximum
  unsigned long long count0 = 0;
  {
    uint32_t zero;
    asm volatile("v_mov_b32 %0, 0" : "=v"(zero));   // (a lane offset the compiler cannot see through: the word travels with the loads below)
    count0 = __hip_atomic_load(cnt + my_group + zero, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  const uint32_t max_seen = read_max_bits(g, t);
  const StepTable* mine = tab + b;
  float total;
  double mass;
  // where this workgroup's run of samples starts, to within a few: the mass in front of node b over seg
  auto window_start = [&](double m) -> uint32_t {
    const double est = m * (double)B;   // (the division is done where the table is built: it would stand in front of this workgroup's second trip)
    const uint32_t s_guess = est >= (double)B ? B : (est > 0.0 ? (uint32_t)est : 0u);   // (not a number: 0)
    return s_guess > kStepPad ? s_guess - kStepPad : 0u;
  };
  [[maybe_unused]] float early_u = 0.0f, early_prio = 0.0f;
  if constexpr (STATIC) {
    total = pre_total;
    mass = pre_mass;
    if (tid < n_steps) path[tid] = pre_path;
    // the window's inputs are asked for here, together with the subtree's heights: the entry that says where the
    // window lies came in beside the arguments
    const uint32_t sw = window_start(mass) + tid;
    if (sw < B) {
      early_u = rng.on ? 0.0f : u[(size_t)t * B + sw];
      early_prio = upd_prio[(size_t)t * B + sw];
    }
  } else {
    total = mine->total;
    mass = mine->mass;
    if (tid < n_steps) path[tid] = mine->path[tid];
  }
#pragma unroll
  for (int i = 0; i < kStepSub; ++i) {
    if (i < n_sub) {
      const uint32_t first = b * sh.sub_cnt[i];       // first node of height 1 + i under b
      const float* src = sh.sub_ptr[i] + (size_t)t * sh.sub_stride[i];
      for (uint32_t e = tid; e < sh.sub_cnt[i]; e += BD)
        sub[sh.sub_off[i] + e] = first + e < sh.sub_pad[i] ? src[first + e] : 0.0f;
    }
  }
  const unsigned long long calls = count0 / owners_of_group(sh.owners, my_group);
  const uint32_t par = (uint32_t)calls & 1u;          // which set of slots and builder counters this call uses
  __syncthreads();
  PER_MARK(1);
  const bool leader = b == 0 && tid == 0;

  // This owner is done: one more in its group's counter (no answer is waited for).
  auto count_me_in = [&]() {
    __syncthreads();   // every lane of the workgroup has issued its stores
    if (tid == 0) atomicAdd(sh.cnt + (size_t)t * kStepGroups + my_group, 1ull);
  };
  // TAIL: the same with an answer: the last owner of a group announces the group, the last group ends the call.
  auto arrive = [&]() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");   // (each wave waits for its stores and atomics to complete)
    __syncthreads();
    if (wave == 0) {
      uint32_t last = 0;
      if (lane == 0) {
        const uint32_t members = owners_of_group(sh.owners, my_group);
        const unsigned long long old = atomicAdd(sh.cnt + (size_t)t * kStepGroups + my_group, 1ull);
        if (old + 1ull == (calls + 1ull) * members) {
          const uint32_t n_groups = sh.owners < kStepGroups ? sh.owners : kStepGroups;
          const unsigned long long old2 = atomicAdd(sh.cnt2 + t, 1ull);
          last = (old2 + 1ull) % n_groups == 0ull ? 1u : 0u;
        }
      }
      if (__shfl((int)last, 0)) {
        // every helper must have read the call's number before it changes (they say so when they have; bounded wait;
        // the slots are read side by side, one per lane)
        const uint32_t* slot = sh.done + ((size_t)t * 2 + par) * kStepDoneSlots;
        uint32_t spins = 0;
        bool ok = true;
        for (;;) {
          uint32_t d = lane < kStepDoneSlots ? __hip_atomic_load(slot + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0u;
#pragma unroll
          for (int m = 1; m < (int)kStepDoneSlots; m <<= 1) d += (uint32_t)__shfl_xor((int)d, m);
          if (__shfl((int)d, 0) >= (int)sh.helpers) break;
          if (++spins > kStepSpinLimit) {
            ok = false;
            break;
          }
          __builtin_amdgcn_s_sleep(2);
        }
        if (lane == 0) {
          if (!ok) atomicOr(&g.status[t], 8u);
          __hip_atomic_store(sh.rel + t, (uint32_t)calls + 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
      }
    }
  };
  // The words of the next call's parity start empty (nothing of this call touches them).
  auto arm_next_call = [&]() {
    if (b != 0) return;
    for (uint32_t i = tid; i < kVminSlots; i += BD) sh.vmin[((size_t)t * 2 + (par ^ 1u)) * kVminSlots + i] = 0x7F800000u;
    if (tid < kStepDoneSlots) sh.done[((size_t)t * 2 + (par ^ 1u)) * kStepDoneSlots + tid] = 0u;
  };
  // Waits (bounded) until every builder workgroup has recorded its elements.  The builders come first in the grid
  // and wait for nothing, so the wait ends; a workgroup that gives up says so in the status word.
  auto wait_for_builders = [&]() -> bool {
    if (!sh.builders) return true;
    if (wave == 0) {
      uint32_t spins = 0, ok = 1;
      const uint32_t* slot = sh.done + ((size_t)t * 2 + par) * kStepDoneSlots;
      for (;;) {
        uint32_t d = lane < kStepDoneSlots ? __hip_atomic_load(slot + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0u;
#pragma unroll
        for (int m = 1; m < (int)kStepDoneSlots; m <<= 1) d += (uint32_t)__shfl_xor((int)d, m);
        if (__shfl((int)d, 0) >= (int)(TAIL ? sh.helpers : sh.builders)) break;
        if (++spins > kStepSpinLimit) {
          ok = 0;
          break;
        }
        __builtin_amdgcn_s_sleep(4);
      }
      if (lane == 0) {
        s_u32[0] = ok;
        if (!ok) atomicOr(&g.status[t], 8u);
      }
    }
    __syncthreads();
    const bool ok = s_u32[0] != 0;
    __syncthreads();
    return ok;
  };
  if (!(total > 0.0f)) {   // nothing can be sampled from this tree; workgroup b reports a slice of the batch
    const bool waited = wait_for_builders();
    const uint32_t share = (B + sh.owners - 1u) / sh.owners;   // (a contiguous share: its rows are this workgroup's too)
    const uint32_t s_lo = b * share < B ? b * share : B, s_hi = s_lo + share < B ? s_lo + share : B;
    for (uint32_t s = s_lo + tid; s < s_hi; s += BD) {
      const size_t o = (size_t)t * B + s;
      out_idx[o] = 0xFFFFFFFFu;
      if (out_prio) out_prio[o] = 0.0f;
      if (out_w) out_w[o] = 0.0f;
      if (sh.builders && waited) inv[s] = 0u;   // (what the builders have recorded goes unused: no element is valid)
    }
    // (without a map every element is out of range too; with one the builders have said so)
    if (leader) atomicOr(&g.status[t], sh.builders && !(TAIL && tail_has_rows) ? 4u : 5u);   // (rows of an index out of range: flag 1)
    // (every owner leaves its node's value: whoever builds the next tables takes all of them)
    if (tid == 0) __hip_atomic_store(&side_ho[b], mine->node, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    arm_next_call();
    if constexpr (TAIL) {
      arrive();
      for (uint32_t f = 0; f < tail.ft.n_fields; ++f) {   // (rows of zeros; the flag that says why is set above)
        if (!tail.ft.io[f]) continue;
        uint8_t* dst = tail.ft.io[f] + ((size_t)t * B + s_lo) * tail.ft.bytes[f];
        for (size_t i = tid; i < (size_t)(s_hi - s_lo) * tail.ft.bytes[f]; i += BD) dst[i] = 0;
      }
    } else {
      count_me_in();
    }
    return;
  }
  const float seg = total / (float)B;

  // where a target lands relative to node b: 0 in front of it, 1 in its subtree (r then holds what is left of the
  // target inside it), 2 behind it.  The same comparisons and subtractions as the walk through the child groups.
  auto landing = [&](float& r) -> uint32_t {
    uint32_t res = 1u;
    bool open = true;   // still on the way to b
    for (int lv = 0; lv < n_top; ++lv) {   // the steps inside one child group: their table entries are read together
      float2 e[LOGK];
#pragma unroll
      for (int j = 0; j < LOGK; ++j) {
        if constexpr (STATIC) {   // (the entries sit in the lanes of every wave: read from there, they are scalars)
          e[j].x = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(pre_path.x), lv * LOGK + j));
          e[j].y = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(pre_path.y), lv * LOGK + j));
        } else {
          e[j] = path[lv * LOGK + j];
        }
      }
#pragma unroll
      for (int j = 0; j < LOGK; ++j) {   // (selects, no early way out: lanes that leave at different steps made the steps cost a branch each)
        // The step's facts are the same for every lane: whether b lies to the right (want), and the left block's sum,
        // taken as infinite for the comparison when the right block is zero (nobody goes right then) and as zero for
        // the subtraction when b lies to the left (lanes still on b's way keep their target; the others' is not used).
        const uint32_t fl = __float_as_uint(e[j].y);
        const bool want = (fl & 1u) != 0u;
        const float L_cmp = (fl & 2u) ? e[j].x : __builtin_huge_valf();
        const float L_sub = want ? e[j].x : 0.0f;
        const bool stay = !(r < L_cmp) == want;
        res = open && !stay ? (want ? 0u : 2u) : res;
        open = open && stay;
        r = r - L_sub;
      }
    }
    return res;
  };
  auto uniform_of = [&](uint32_t s) -> float { return rng.on ? counter_uniform(rng, s, t) : u[(size_t)t * B + s]; };
  auto landing_of = [&](uint32_t s) -> uint32_t {   // (samples beyond the batch: behind every node)
    if (!(s < B)) return 2u;
    float r = ((float)s + uniform_of(s)) * seg;
    return landing(r);
  };
  // smallest s in [0, B] whose sample lands at or behind b (level 1) or behind it (level 2); one wave, 64 probes per round
  auto first_at = [&](uint32_t level) -> uint32_t {
    uint32_t lo = 0, hi = B;
    while (lo < hi) {
      const uint32_t span = hi - lo, stride = (span + 63u) / 64u;
      const uint64_t s64 = (uint64_t)lo + (uint64_t)lane * stride;
      const bool probe = s64 < hi;
      const bool ge = !probe || landing_of((uint32_t)s64) >= level;
      const unsigned long long m = __ballot(ge);
      if (m == 0ull) {
        lo = lo + 63u * stride + 1u;
      } else {
        const uint32_t f = (uint32_t)__ffsll((long long)m) - 1u;
        const uint64_t at = (uint64_t)lo + (uint64_t)f * stride;
        if (f > 0) lo = lo + (f - 1u) * stride + 1u;
        if (at < hi) hi = (uint32_t)at;
      }
    }
    return lo;
  };

  const uint32_t s0 = window_start(mass);
  PER_MARK(3);

  // ---- trip 2: the samples of the window [s0, s0 + BD): uniforms, their own new priorities
  uint32_t s = s0 + tid;
  const bool in = s < B;
  float u_s, prio_s;
  if constexpr (STATIC) {
    u_s = in ? (rng.on ? uniform_of(s) : early_u) : 0.0f;
    prio_s = in ? early_prio : 0.0f;
  } else {
    u_s = in ? uniform_of(s) : 0.0f;
    prio_s = in ? upd_prio[(size_t)t * B + s] : 0.0f;
  }
  float r = ((float)s + u_s) * seg, val = total;
  PER_MARK(2);
  const uint32_t where = in ? landing(r) : 2u;
  PER_MARK(14);
  // does the window hold the whole run?  its first sample must land in front of b (or be sample 0), and a sample
  // of it must land behind b (or the batch must end in it)
  uint32_t run_lo, run_n;
  bool searched;   // (uniform over the workgroup)
  {
    if (tid == 0) s_u32[1] = (s0 == 0 || where == 0u) ? 1u : 0u;
    const uint32_t n_front = (uint32_t)__syncthreads_count(in && where == 0u);
    const uint32_t n_mine = (uint32_t)__syncthreads_count(in && where == 1u);
    const bool complete = s_u32[1] != 0 && (n_front + n_mine < BD || s0 + BD >= B);
    run_lo = s0 + n_front;
    run_n = n_mine;
    if (!complete) {   // rare: the exact ends of the run by search, then chunks of it (uniform over the workgroup)
      if (wave == 0) {
        const uint32_t lo = first_at(1u), hi = first_at(2u);
        if (lane == 0) {
          s_u32[2] = lo;
          s_u32[3] = hi;
        }
      }
      __syncthreads();
      run_lo = s_u32[2];
      run_n = s_u32[3] - s_u32[2];
    }
    searched = !complete;
  }
  const uint32_t n_chunks = searched ? (run_n + BD - 1u) / BD : 1u;
  const bool two_phase = n_chunks > 1;
  PER_MARK(4);

  const uint32_t lo1 = b * sh.sub_cnt[0];                                   // first height-1 node of the subtree
  float* leaves = g.level[0] + (size_t)t * g.stride[0];
  float* lvl1 = sh.sub_ptr[0] + (size_t)t * sh.sub_stride[0];
  float* stage = c.rows + (size_t)(1u + wave * 64u) * ROW;                  // this wave's rows: slots 1 + tid
  uint32_t mx = 0, flags = 0, vmin_bits = 0x7F800000u;
  bool builders_ok = true, waited = false;
  if (tid == 0) {
    c.key[0] = kNoKey;
    c.wpos[0] = 0;
    c.touch[0] = 0;
  }
  if (tid < 2) c.key[BD + tid] = kNoKey;   // (key[BD] is written again by the last lane; key[BD + 1] stays)

  for (uint32_t pass = 0; pass < (two_phase ? 2u : 1u); ++pass) {
    // pass 0 walks (and, when one chunk holds the run, updates); pass 1 of a long run updates chunk by chunk
    for (uint32_t ch = 0; ch < n_chunks; ++ch) {
      bool member;
      uint32_t idx = kNoKey;
      if (searched) {
        s = run_lo + ch * BD + tid;
        member = s < run_lo + run_n;
        if (pass == 0) {
          u_s = member ? uniform_of(s) : 0.0f;
          r = ((float)s + u_s) * seg;
          val = total;
          (void)landing(r);
        }
        prio_s = member ? upd_prio[(size_t)t * B + s] : 0.0f;
      } else {
        member = in && where == 1u;
      }
      const size_t o = (size_t)t * B + (member ? s : 0u);
      uint32_t x = b;   // node of height ho
      if (pass == 0) {
        // ---- the own subtree's heights from LDS
        if (!member) r = 0.0f;
#pragma unroll
        for (int i = kStepSub - 1; i >= 0; --i) {
          if (i < n_sub) {
            const uint32_t local = x - b * (sh.sub_cnt[i] >> LOGK);   // x - first node of height 2 + i under b
            unsigned child;
            descend_lane<LOGK>(sub + sh.sub_off[i] + (size_t)local * K, r, child, val);
            x = x * K + child;
          }
        }
      } else {
        idx = member ? out_idx[o] : kNoKey;
        x = member ? idx >> LOGK : lo1;
      }
      // ---- trip 3: the leaf groups, staged row by row
      __syncthreads();   // (the rows of the chunk before are no longer read)
      stage_groups<LOGK, 0>(leaves, x, lane, stage);
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      if (pass == 0) {
        unsigned child;
        descend_lane<LOGK>(stage + lane * ROW, r, child, val);
        idx = x * K + child;
        if (member) {
          out_idx[o] = idx;
          if (out_prio) out_prio[o] = val;
          if (out_w) out_w[o] = val;
          const uint32_t vb = __float_as_uint(val);
          vmin_bits = vb < vmin_bits ? vb : vmin_bits;
        }
        if (two_phase) continue;
      }
      PER_MARK(5);
      // ---- the update of this chunk
      if (!waited) {
        builders_ok = wait_for_builders();
        waited = true;
      }
      uint32_t w = 0;
      float wv = 0.0f;
      if (member) {
        if (!(idx < size)) {
          flags |= 1u;
          if (sh.builders && builders_ok) (void)atomicExch(&inv[s], 0u);
        } else if (sh.builders) {
          if (builders_ok) {
            w = atomicExch(&inv[s], 0u);
            if (w) wv = w == s + 1u ? prio_s : upd_prio[(size_t)t * B + (w - 1u)];
          }
        } else if (valid_priority(prio_s)) {
          w = s + 1u;
          wv = prio_s;
          const uint32_t vb = wv > 0.0f ? __float_as_uint(wv) : 0u;
          mx = vb > mx ? vb : mx;
        } else {
          flags |= 2u;
        }
      }
      c.key[1 + tid] = member ? idx : kNoKey;
      c.wpos[1 + tid] = w;
      c.wval[1 + tid] = wv;
      c.touch[1 + tid] = 0u;
      PER_MARK(6);
      const bool last_chunk = ch + 1 == n_chunks;
      __syncthreads();
      uint32_t open_pos = 0;
      float open_val = 0.0f;
      chunk_leaves<LOGK>(c, tid, BD, last_chunk, leaves, open_pos, open_val);
      if (tid == 0) chunk_leaves<LOGK>(c, BD, BD, last_chunk, leaves, open_pos, open_val);
      __syncthreads();
      uint32_t open_head = chunk_groups<LOGK>(c, tid, BD, last_chunk, lvl1, sub + sh.sub_off[0], lo1);
      if (tid == 0) open_head = chunk_groups<LOGK>(c, BD, BD, last_chunk, lvl1, sub + sh.sub_off[0], lo1);
      __syncthreads();
      PER_MARK(7);
      if (!last_chunk) {   // what stays open moves to slot 0 (thread 0 has worked on slot BD)
        if (tid == 0) {
          s_u32[4] = open_head;
          s_u32[5] = c.key[BD];
          s_u32[6] = open_pos;
          s_u32[7] = __float_as_uint(open_val);
        }
        __syncthreads();
        const uint32_t h = s_u32[4];
        float carry = 0.0f;
        if (h != kNoKey && tid < (uint32_t)K) carry = c.rows[(size_t)h * ROW + tid];
        const uint32_t touched = h != kNoKey ? c.touch[h] : 0u;
        __syncthreads();
        if (h != kNoKey && tid < (uint32_t)K) c.rows[tid] = carry;
        if (tid == 0) {
          c.key[0] = h != kNoKey ? s_u32[5] : kNoKey;
          c.wpos[0] = s_u32[6];
          c.wval[0] = __uint_as_float(s_u32[7]);
          c.touch[0] = touched;
        }
      }
    }
    if (pass == 0 && two_phase) __syncthreads();   // the indices written above are read back by the second pass
  }

  // ---- the heights 2 .. ho-1 of the subtree and node b itself, from LDS; what changed is stored
  __syncthreads();
  {
    const unsigned q = tid % LPS;
    const uint32_t grp = tid / LPS, ngrp = BD / LPS;
#pragma unroll
    for (int i = 1; i < kStepSub; ++i) {
      if (i < n_sub) {
        const uint32_t first = b * sh.sub_cnt[i];
        float* dst = sh.sub_ptr[i] + (size_t)t * sh.sub_stride[i];
        for (uint32_t base = 0; base < sh.sub_cnt[i]; base += ngrp) {
          const uint32_t e = base + grp;
          const bool ok = e < sh.sub_cnt[i];
          const float sum = group_sum<LOGK>(sub + sh.sub_off[i - 1] + (size_t)(ok ? e : 0u) * K, q);
          if (ok && q == 0) {
            float* mine = sub + sh.sub_off[i] + e;
            if (__float_as_uint(*mine) != __float_as_uint(sum)) {
              *mine = sum;
              dst[first + e] = sum;
            }
          }
        }
        __syncthreads();
      }
    }
    // node b: the sum of its K children, the nodes of height ho-1 of the subtree
    uint32_t off_last = sh.sub_off[0];
#pragma unroll
    for (int i = 1; i < kStepSub; ++i)
      if (i == n_sub - 1) off_last = sh.sub_off[i];
    if (tid < 64) {
      const float sum = group_sum<LOGK>(sub + off_last, lane % LPS);
      if (lane == 0) __hip_atomic_store(&side_ho[b], sum, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // (past the caches: read by another workgroup of this kernel when the call ends in it)
    }
  }
  PER_MARK(8);
  // ---- running maximum, flags, the smallest sampled value of this workgroup
  if (!sh.builders) raise_max(g, t, mx, max_seen);
  if (flags) atomicOr(&g.status[t], flags);
  arm_next_call();
  PER_MARK(9);
  PER_FLUSH();
  if (out_w) {   // the smallest value this workgroup has sampled, for the kernel that turns the values into weights
    const uint32_t m = wave_min_u32(vmin_bits);
    if (lane == 0 && m != 0x7F800000u)
      atomicMin(sh.vmin + ((size_t)t * 2 + par) * kVminSlots + (b * (BD >> 6) + wave) % kVminSlots, m);
  }
  if constexpr (!TAIL) {
    count_me_in();
  } else {
    arrive();
    PER_MARK(10);
    // the rows of this owner's own samples, while the other owners arrive
    for (uint32_t f = 0; f < tail.ft.n_fields; ++f) {   // (a loop, not unrolled: the movers' code once)
      if (!tail.ft.io[f]) continue;
      if (tail.ft.vec[f] == 16) {
        // fields that move in 16-byte pieces: four pieces per lane in flight, all loads before the first store; the
        // index of a row comes from LDS where the run was one window (its lanes have left them there)
        const uint32_t E = tail.ft.bytes[f], epr = E / 16u, RS = tail.ft.row_stride;
        const uint32_t total_e = run_n * epr;
        const uint8_t* col = tail.ft.col[f] + (uint64_t)t * tail.ft.col_stride[f];
        uint8_t* io = tail.ft.io[f] + ((uint64_t)t * B + run_lo) * E;
        bool bad = false;
        for (uint32_t e0 = tid; e0 < total_e; e0 += 4u * BD) {
          uint4 v[4];
#pragma unroll
          for (int k = 0; k < 4; ++k) {
            const uint32_t e = e0 + (uint32_t)k * BD;
            const bool live = e < total_e;
            const uint32_t row = live ? e / epr : 0u, piece = e % epr;
            const uint32_t at = searched ? out_idx[(size_t)t * B + run_lo + row] : c.key[1u + (run_lo - s0) + row];
            const bool ok = at < g.N;
            bad = bad || (live && !ok);
            v[k] = *reinterpret_cast<const uint4*>(col + (uint64_t)(ok ? at : 0u) * RS + piece * 16u);
            if (!ok) v[k] = make_uint4(0, 0, 0, 0);
          }
#pragma unroll
          for (int k = 0; k < 4; ++k) {
            const uint32_t e = e0 + (uint32_t)k * BD;
            if (e < total_e) *reinterpret_cast<uint4*>(io + (uint64_t)e * 16u) = v[k];
          }
        }
        if (bad) atomicOr(&g.status[t], 1u);
      } else {
        rows_job<true, false>(tail.ft, f, t, B, out_idx, 0, g.N, g.status, 0, 1, run_lo, run_n);
      }
    }
    PER_MARK(11);
    const bool released = out_w && wait_release((uint32_t)calls + 1u);
    PER_MARK(12);
    if (released) {
      // the batch's smallest sampled value: every owner's contribution is in the slots now
      const uint32_t* slots = sh.vmin + ((size_t)t * 2 + par) * kVminSlots;
      uint32_t m = 0x7F800000u;
      for (uint32_t i = tid; i < kVminSlots; i += BD) m = min_u32(m, __hip_atomic_load(slots + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
      m = wave_min_u32(m);
      if (lane == 0) s_u32[wave] = m;
      __syncthreads();
      for (uint32_t wv = 0; wv < (BD >> 6); ++wv) m = min_u32(m, s_u32[wv]);
      if (weight_mode & kWeightBufferNorm) m = buffer_min_bits(g, t, weight_mode);
      for (uint32_t i = tid; i < run_n; i += BD) {
        const size_t o = (size_t)t * B + run_lo + i;
        out_w[o] = importance_weight(out_w[o], __uint_as_float(m), beta);
      }
    }
    PER_MARK(13);
    PER_FLUSH_TAG(2);
  }
}

// The tables of the owners [first, first + count) of tree t from the nodes of height ho at src (the level array, or
// the side array the owners of a call have just filled), by one workgroup; dynamic LDS holds the heights ho .. H-1.
// The workgroup with first == 0 also puts the tree's memory in order: the level array of height ho takes src's values
// (if src is the side array) and the heights above are recomputed and stored, so that nothing is left stale.
// COHERENT: src was written by other workgroups of the running kernel (with device-scope atomic stores) and is read
// the same way.
template <int LOGK, bool COHERENT>
__device__ __forceinline__ void build_tables(const StepShape& sh, uint32_t t, const float* src, bool from_side, uint32_t first,
                                             uint32_t count, float* top, float* skipped) {
  constexpr int K = Fan<LOGK>::K;
  constexpr int LPS = Fan<LOGK>::LPS;
  const uint32_t tid = threadIdx.x, BD = blockDim.x;
  const int n_top = (int)sh.n_top;
  for (uint32_t i = tid; i < sh.top_cnt[0]; i += BD) {
    float v = 0.0f;
    if (i < sh.top_n[0]) v = COHERENT ? __hip_atomic_load(src + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : src[i];
    top[sh.top_off[0] + i] = v;
  }
  __syncthreads();
  {
    const unsigned q = tid % LPS;
    const uint32_t grp = tid / LPS, ngrp = BD / LPS;
#pragma unroll
    for (int i = 1; i < kStepTop; ++i) {
      if (i < n_top) {
        for (uint32_t base = 0; base < sh.top_cnt[i]; base += ngrp) {
          const uint32_t j = base + grp;
          const bool real = j < sh.top_n[i];
          const float sum = group_sum<LOGK>(top + sh.top_off[i - 1] + (size_t)(real ? j : 0u) * K, q);
          if (q == 0 && j < sh.top_cnt[i]) top[sh.top_off[i] + j] = real ? sum : 0.0f;
        }
        __syncthreads();
      }
    }
  }
  const float* rootgrp = top;   // group 0 of height H-1
#pragma unroll
  for (int i = 0; i < kStepTop; ++i)
    if (i == n_top - 1) rootgrp = top + sh.top_off[i];
  const float total = row_sum<LOGK>(rootgrp);
  if (first == 0) {   // the tree's memory: height ho, the heights above, the root
    if (from_side) {
      float* lvl = sh.top_ptr[0] + (size_t)t * sh.top_stride[0];
      for (uint32_t i = tid; i < sh.top_n[0]; i += BD) lvl[i] = top[sh.top_off[0] + i];
    }
#pragma unroll
    for (int i = 1; i < kStepTop; ++i) {
      if (i < n_top) {
        float* lvl = sh.top_ptr[i] + (size_t)t * sh.top_stride[i];
        for (uint32_t j = tid; j < sh.top_n[i]; j += BD) lvl[j] = top[sh.top_off[i] + j];
      }
    }
    if (tid == 0) sh.root[(size_t)t * sh.root_stride] = total;
  }
  StepTable* tab = sh.tab + (size_t)t * sh.owners;
  const uint32_t n_steps = (uint32_t)n_top * LOGK;
  // one binary step of one owner per lane: step k halves the block of the child group of height ho + i that holds the
  // owner's ancestor (i = n_top-1 first) and notes the sums of the two halves, in the order of the walk inside a group
  for (uint32_t item = tid; item < count * n_steps; item += BD) {
    const uint32_t b = first + item / n_steps, k = item % n_steps;
    const uint32_t i = (uint32_t)n_top - 1u - k / LOGK, m = LOGK - 1u - k % LOGK;   // height ho + i; halves of 2^m nodes
    uint32_t off_i = sh.top_off[0];
#pragma unroll
    for (int kk = 1; kk < kStepTop; ++kk)
      if ((uint32_t)kk == i) off_i = sh.top_off[kk];
    const uint32_t anc = shr64(b, i * LOGK);                 // the owner's ancestor at height ho + i
    const uint32_t pos = anc & (uint32_t)(K - 1);
    const float* blk = top + off_i + (size_t)(anc - pos) + ((pos >> (m + 1)) << (m + 1));
    const float left = block_sum<LOGK>(blk, m), right = block_sum<LOGK>(blk + (1u << m), m);
    const uint32_t turn = (pos >> m) & 1u;
    tab[b].path[k] = make_float2(left, __uint_as_float(turn | (right != 0.0f ? 2u : 0u)));
    skipped[item] = turn ? left : 0.0f;
  }
  __syncthreads();
  // the mass in front of every owner's node: the left blocks its way from the root passes by (only used to guess
  // where its run of samples starts); its own value; the total
  for (uint32_t e = tid; e < count; e += BD) {
    const uint32_t b = first + e;
    double mass = 0.0;
    for (uint32_t k = 0; k < n_steps; ++k) mass += (double)skipped[e * n_steps + k];
    tab[b].mass = total > 0.0f ? mass / (double)total : 0.0;
    tab[b].total = total;
    tab[b].node = top[sh.top_off[0] + b];
  }
}

// In front of a step when another call has changed the tree since the tables were built.
template <int LOGK>
__global__ void __launch_bounds__(256)
k_step_tables(StepShape sh) {
  extern __shared__ __attribute__((aligned(16))) float top[];
  const uint32_t t = blockIdx.y, first = blockIdx.x * kTableOwners;
  const uint32_t count = sh.owners - first < kTableOwners ? sh.owners - first : kTableOwners;
  __shared__ float skipped[kTableOwners * kStepPathMax];
  build_tables<LOGK, false>(sh, t, sh.top_ptr[0] + (size_t)t * sh.top_stride[0], false, first, count, top, skipped);
}

// Ends a step: the first table_blocks workgroups take the owners' new nodes of height ho into the tree and build the
// tables of the next call; beside them run the jobs of what is left of the sampling call (JobRanges: job 0 the
// weights, jobs 2 + f the rows of field f): the weights job turns the sampled values the owners have left in w into importance weights
// (the smallest of them sit in the slots of the call's parity; the call that has just finished is number
// finished calls - 1).
template <int LOGK, bool WIDE>
__global__ void __launch_bounds__(256)
k_step_epilogue(Geom g, StepShape sh, uint32_t table_blocks, uint32_t B, float beta, uint32_t weight_mode,
                float* __restrict__ w, const uint32_t* __restrict__ idx, FieldTable ft, JobRanges jr) {
  // (only the lines that the row and weight workgroups read, which are what the kernel waits for: the first words of
  // the geometry, the status and scalar pointers, the counters and minima of the step's shape, and everything from
  // the call's own arguments on: field table, job ranges; the table builders fetch the rest as they go)
  touch_kernel_argument_lines<kStepEpilogueArgLines>();
  extern __shared__ __attribute__((aligned(16))) float top[];
  __shared__ uint32_t s_m[4];
  __shared__ float skipped[kTableOwners * kStepPathMax];
  const uint32_t t = blockIdx.y;
  if (blockIdx.x < table_blocks) {
    const uint32_t first = blockIdx.x * kTableOwners;
    const uint32_t count = sh.owners - first < kTableOwners ? sh.owners - first : kTableOwners;
    build_tables<LOGK, false>(sh, t, sh.side + (size_t)t * sh.side_stride, true, first, count, top, skipped);
    if (blockIdx.x == 0 && threadIdx.x == 0)   // the number of finished calls, for calls that read it from this word
      sh.rel[t] = (uint32_t)(sh.cnt[(size_t)t * kStepGroups] / owners_of_group(sh.owners, 0));
    return;
  }
  const uint32_t job = blockIdx.x - table_blocks;
  if (job >= jr.first[1]) {   // the rows of the sampled indices, one job per payload field
    const uint32_t f = job_field(jr, job);
    if (f < (uint32_t)kMaxFields)
      rows_job<true, WIDE>(ft, f, t, B, idx, 0, g.N, g.status, job - jr.first[2 + f], jr.first[3 + f] - jr.first[2 + f]);
    return;
  }
  const unsigned long long calls = sh.cnt[(size_t)t * kStepGroups] / owners_of_group(sh.owners, 0);
  const uint32_t par = (uint32_t)(calls - 1ull) & 1u;
  const uint32_t* slots = sh.vmin + ((size_t)t * 2 + par) * kVminSlots;
  const uint32_t i = job * blockDim.x + threadIdx.x;
  const size_t o = (size_t)t * B + (i < B ? i : 0u);
  const float v = w[o];
  uint32_t m = wave_min_u32(slots[threadIdx.x % kVminSlots]);   // (256 lanes: every slot once)
  if ((threadIdx.x & 63u) == 0) s_m[threadIdx.x >> 6] = m;
  __syncthreads();
  m = min_u32(min_u32(s_m[0], s_m[1]), min_u32(s_m[2], s_m[3]));
  const bool nothing_sampled = m == 0x7F800000u;   // (the tree's total was zero: the values are zeros already)
  if (weight_mode & kWeightBufferNorm) m = buffer_min_bits(g, t, weight_mode);
  if (i < B) w[o] = nothing_sampled ? 0.0f : importance_weight(v, __uint_as_float(m), beta);
}

// The owner height of a tree for k_step, or 0 when the kernel does not fit it: the lowest height, not below the
// tree pass's own workgroup roots, with at most 2048 nodes over all trees, whose subtrees (heights 1 .. ho-1)
// and the heights from it to the root are small enough for LDS.
uint32_t step_owner_height(const Geom& g) {
  if (g.logK < 3) return 0;
  for (uint32_t ho = tree_pass_height(g) < 2 ? 2 : tree_pass_height(g); ho + 1 <= g.H; ++ho) {
    if ((uint64_t)g.n[ho] * g.T > kStepMaxOwners || g.n[ho] > kLazyTopNodes) continue;
    if (g.H - ho > (uint32_t)kStepTop || ho - 1 > (uint32_t)kStepSub) return 0;
    uint64_t sub = 0;
    for (uint32_t l = 1; l < ho; ++l) sub += 1ull << ((ho - l) * g.logK);
    if (sub > 16384) return 0;
    return ho;
  }
  return 0;
}
size_t step_table_bytes() { return (size_t)kStepMaxOwners * sizeof(StepTable); }

// Workgroup size for a batch of B samples per tree: room for one and a half times the average run of samples
// per owner, within what the staging rows leave of the LDS; 0 when the runs would be too long for one chunk
// (the separate kernels are the better choice then).
template <int LOGK>
static uint32_t step_block(const Geom& g, uint32_t ho, uint32_t B) {
  constexpr int K = Fan<LOGK>::K;
  const uint32_t most = K >= 32 ? 256u : 512u;
  const uint64_t avg = ((uint64_t)B + g.n[ho] - 1) / g.n[ho];
  const uint64_t want = avg + avg / 2 + 2 * kStepPad + 8;
  if (want > most) return 0;
  const uint32_t block = (uint32_t)((want + 63) / 64 * 64);
  return block < 64 ? 64 : block;
}

// Descriptors of both kernels' views of the tree; *step_lds: dynamic LDS of k_step with this block size; *table_lds: of
// the kernels that build the tables.
template <int LOGK>
static void step_shape(const Geom& g, uint32_t block, uint32_t B, bool with_map, StepShape* out, size_t* step_lds,
                       size_t* table_lds) {
  constexpr int K = Fan<LOGK>::K;
  const uint32_t ho = g.step_ho;
  StepShape sh{};
  sh.n_top = g.H - ho;
  sh.n_sub = ho - 1;
  uint32_t off = 0;
  for (uint32_t i = 0; i < sh.n_top; ++i) {   // (LDS of the table kernels)
    const uint32_t l = ho + i;
    sh.top_ptr[i] = g.level[l];
    sh.top_stride[i] = g.stride[l];
    sh.top_cnt[i] = g.n[l + 1] * K;
    sh.top_n[i] = g.n[l];
    sh.top_off[i] = off;
    off += sh.top_cnt[i];
  }
  *table_lds = (size_t)off * 4;
  off = 0;
  for (uint32_t i = 0; i < sh.n_sub; ++i) {   // (LDS of k_step)
    const uint32_t l = 1 + i;
    sh.sub_ptr[i] = g.level[l];
    sh.sub_stride[i] = g.stride[l];
    sh.sub_cnt[i] = 1u << ((ho - l) * LOGK);
    sh.sub_pad[i] = (uint32_t)(((uint64_t)g.n[l] + K - 1) / K * K);
    sh.sub_off[i] = off;
    off += sh.sub_cnt[i];
  }
  off = (off + 1u) / 2u * 2u;
  sh.path_off = off;
  off += 2u * kStepPathMax;
  off = (off + 3u) / 4u * 4u;
  sh.rows_off = off;
  off += (block + 1u) * (K + 4);
  sh.key_off = off;
  off += (block + 2u) + 3u * (block + 1u);
  sh.owners = g.n[ho];
  sh.builders = 0;
  if (with_map) {
    sh.builders = (B + 4u * block - 1u) / (4u * block);   // about four elements per builder lane
    if (sh.builders > 64) sh.builders = 64;
  }
  sh.root = g.root;
  sh.root_stride = g.root_stride;
  sh.side = g.step_side;
  sh.side_stride = g.step_side_stride;
  sh.tab = reinterpret_cast<StepTable*>(g.step_tab);
  sh.cnt = g.step_cnt;
  sh.done = g.step_done;
  sh.vmin = g.step_vmin;
  sh.inv = reinterpret_cast<uint32_t*>(g.owner);
  sh.inv_stride = 2u * g.owner_stride;
  sh.table_blocks = (sh.owners + kTableOwners - 1u) / kTableOwners;
  sh.helpers = sh.builders > sh.table_blocks ? sh.builders : sh.table_blocks;
  sh.cnt2 = g.step_cnt2;
  sh.rel = g.step_rel;
  *out = sh;
  *step_lds = (size_t)off * 4;
}

// Compute units of `device` (0 if the query fails).
static uint32_t compute_units(int device) {
  static std::atomic<int> known[kMaxDevices];
  if (device < 0 || device >= kMaxDevices) return 0;
  int n = known[device].load(std::memory_order_relaxed);
  if (n == 0) {
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess || n < 0) n = 0;
    known[device].store(n, std::memory_order_relaxed);
  }
  return (uint32_t)n;
}

template <int LOGK>
static hipError_t launch_step_k(const Geom& g, const Tuning& tn, uint32_t block, bool tables_valid, uint32_t B, uint32_t size,
                                float beta, uint32_t weight_mode, const float* u, const RngArgs& rng, uint32_t* out_idx,
                                float* out_prio, float* out_w, const float* upd_prio, const uint32_t* upd_pos,
                                const FieldTable* rows, hipStream_t s) {
  StepShape sh;
  size_t bytes, table_bytes;
  step_shape<LOGK>(g, block, B, upd_pos != nullptr, &sh, &bytes, &table_bytes);
  FieldTable ft{};
  if (rows) ft = *rows;
  const bool wide = any_field_moves_wide(rows ? &ft : nullptr);
  // The call ends inside k_step when every workgroup of its grid can be resident at once (its workgroups wait for
  // each other at the end, and one that waits keeps its place).
  bool tail = tn.step_tail && !wide;
  const size_t tail_bytes = bytes > table_bytes ? bytes : table_bytes;
  hipError_t e;
  if (tail) {
    e = grant_lds<&k_step<LOGK, true>>(tn, tail_bytes);
    if (e != hipSuccess) return e;
    int per_cu = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k_step<LOGK, true>, (int)block, tail_bytes) != hipSuccess) per_cu = 0;
    const uint64_t room = (uint64_t)(per_cu > 0 ? per_cu : 0) * compute_units(tn.device);
    tail = (uint64_t)(sh.helpers + sh.owners) * g.T <= room;
  }
  if (!tail) {
    e = grant_lds<&k_step<LOGK, false>>(tn, bytes);
    if (e != hipSuccess) return e;
  }
  if (!tables_valid) {
    PER_LAUNCH(KID_STEP_TABLES, k_step_tables<LOGK>, dim3(sh.table_blocks, g.T), dim3(256), table_bytes, s, sh);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  if (tail) {
    StepTail tl{};
    tl.ft = ft;
    PER_LAUNCH(KID_STEP, (k_step<LOGK, true>), dim3(sh.helpers + sh.owners, g.T), dim3(block), tail_bytes, s, g, sh, B, size, beta,
               weight_mode, u, rng, out_idx, out_prio, out_w, upd_prio, upd_pos, tl);
    return hipGetLastError();
  }
  if (g.step_tab_static && g.T == 1) {   // (the tables sit in the static array: owners fetch their entry beside the arguments)
    e = grant_lds<&k_step<LOGK, false, true>>(tn, bytes);
    if (e != hipSuccess) return e;
    PER_LAUNCH(KID_STEP, (k_step<LOGK, false, true>), dim3(kStepFront + sh.owners, 1), dim3(block), bytes, s, g, sh, B, size, beta,
               weight_mode, u, rng, out_idx, out_prio, out_w, upd_prio, upd_pos, NoTail{});
  } else {
    const dim3 grid(sh.builders + sh.owners, g.T);
    PER_LAUNCH(KID_STEP, (k_step<LOGK, false>), grid, dim3(block), bytes, s, g, sh, B, size, beta, weight_mode, u, rng, out_idx,
               out_prio, out_w, upd_prio, upd_pos, NoTail{});
  }
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  const JobRanges jr = job_ranges(rows ? &ft : nullptr, B, 256, out_w ? B : 0u, 0u, g.T);
  const dim3 egrid(sh.table_blocks + jr.first[2 + kMaxFields], g.T);
  if (wide) {
    PER_LAUNCH(KID_STEP_EPILOGUE, (k_step_epilogue<LOGK, true>), egrid, dim3(256), table_bytes, s, g, sh, sh.table_blocks, B, beta,
               weight_mode, out_w, out_idx, ft, jr);
  } else {
    PER_LAUNCH(KID_STEP_EPILOGUE, (k_step_epilogue<LOGK, false>), egrid, dim3(256), table_bytes, s, g, sh, sh.table_blocks, B, beta,
               weight_mode, out_w, out_idx, ft, jr);
  }
  return hipGetLastError();
}

// Block size k_step would run a batch of B with, 0 when it does not take that batch (or that tree).  `always`
// (a tuning value for tests) lifts the limits that are there for speed only: the kernel pays off for long runs
// of samples per owner on few trees (measured: 65536 samples on one tree of 2^24 leaves 21 against 28 us per
// step; batches of 32 .. 4096, or 64 trees with an insert between the steps, are faster as separate kernels).
uint32_t step_fits(const Geom& g, uint32_t B, bool always) {
  if (!g.step_ho || B == 0 || (uint64_t)B > 2ull * g.owner_stride) return 0;
  // (and for batches of 32768 and more over all trees: 16384 samples on 2^20 leaves at K = 16, 64 per owner, take
  // 11.4 us as separate kernels and 13.4 in this form)
  if (!always && (g.T > 8 || (uint64_t)B < 64ull * g.n[g.step_ho] || (uint64_t)B * g.T < 32768)) return 0;
  switch (g.logK) {
    case 3: return step_block<3>(g, g.step_ho, B);
    case 4: return step_block<4>(g, g.step_ho, B);
    case 5: return step_block<5>(g, g.step_ho, B);
    case 6: return step_block<6>(g, g.step_ho, B);
    default: return 0;
  }
}

// The whole step: [the tables, when tables_valid says they are not current], k_step, the epilogue.  Afterwards the
// tree's memory is in order at every height and the tables are current.
hipError_t launch_step(const Geom& g, const Tuning& tn, uint32_t block, bool tables_valid, uint32_t B, uint32_t size,
                       float beta, const float* u, const RngArgs& rng, uint32_t* out_idx, float* out_w, float* out_prio,
                       uint32_t weight_mode, const FieldTable* rows, const float* upd_prio, const uint32_t* upd_pos,
                       hipStream_t s) {
#define CALL(L) launch_step_k<L>(g, tn, block, tables_valid, B, size, beta, weight_mode, u, rng, out_idx, out_prio, out_w, upd_prio, upd_pos, rows, s)
  switch (g.logK) {
    case 3: return CALL(3);
    case 4: return CALL(4);
    case 5: return CALL(5);
    case 6: return CALL(6);
    default: return hipErrorInvalidValue;
  }
#undef CALL
}
