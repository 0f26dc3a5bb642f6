// chain.hip -- chain runtime and C ABI of libpygraph_hip (see include/pygraph_hip.h).
//
// A chain is a linear kernel-launch DAG.  The runtime keeps, per kernel, three argument blocks:
// one for eager launches (external operands patched with the caller's pointers on every call),
// one whose external operands are static placeholders (graph + copy refresh), and one whose
// external operands are pointer-table slots (graph + Parameter Indirection).  Graphs are made by
// stream capture, once per segment and per graph mode.  A fourth block serves the graphs whose
// kernel nodes are rewritten from the host before each launch (pg_replay_update); those graphs are
// built node by node, so that the runtime keeps a handle on every node.
#include "../../include/pygraph_hip.h"
#include "../../include/pygraph_hip_bench.h"
#include "kernels.h"

#include <hip/hip_ext.h>

#include <algorithm>
#include <chrono>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <string>
#include <vector>

namespace {

thread_local std::string g_err;
thread_local int g_hip_err = 0;

pg_status fail(pg_status st, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_err = buf;
    return st;
}

#define PG_HIP(call)                                                                               \
    do {                                                                                           \
        hipError_t e_ = (call);                                                                    \
        if (e_ != hipSuccess) {                                                                    \
            g_hip_err = (int)e_;                                                                   \
            return fail(PG_EHIP, "%s failed: %s", #call, hipGetErrorString(e_));                   \
        }                                                                                          \
    } while (0)

constexpr size_t kAlign = 256;
constexpr size_t kNoShadow = ~(size_t)0;
size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }
size_t elem_bytes(int dtype) { return dtype == PG_F32 ? 4 : 2; }

union ArgBlock {
    pgk::EwArgs ew;
    pgk::RmsArgs rms;
    pgk::GemvArgs gemv;
    pgk::SbrArgs sbr;
    // every block starts with: out, in0, in1, (in2)
    const void* ptr[4];
};

struct KernelRec {
    pgk::Launch direct, indirect;   // same shape, different kernel variant
    ArgBlock a_eager, a_copy, a_ind, a_upd;
    ArgBlock a_host[2];             // external operands are slots of the two host-resident tables (PG_TABLE_HOST)
    int n_in = 0;
    int ind_mask = 0;               // operands that are external
    int ext_of[3] = {-1, -1, -1};
};

struct CopyList {                   // one refresh job: a set of external tensors -> placeholders
    std::vector<int> ext;           // external indices, ascending
    std::vector<pgk::CopyTensor> tensors;
    std::vector<pgk::CopyChunk> chunks;     // sorted by tensor
    struct Group { int t0, t1, c0, c1; };   // tensors [t0,t1) of this list <-> chunks [c0,c1)
    std::vector<Group> groups;
    size_t tensors_off = 0, chunks_off = 0; // in the workspace
    long long bytes = 0;
};

// A run of consecutive kernels of one segment that a captured graph plays with one dispatch
// (kernels.h, "merged dispatches").  Runs of one kernel are launched as that kernel.
struct MergeGroup {
    int k0 = 0, k1 = 0;              // kernels [k0, k1)
    bool head = false;               // the run is a GEMV's dispatch: the kernels after the GEMV ride in it as an epilogue
    bool pro = false;                // (head) kernel k0 is the RMSNorm that feeds the GEMV k0 + 1, and rides in front of it as a prologue
    int rename = -1;                 // (pro) internal buffer the RMSNorm reads and the run overwrites: the run writes its other copy
    bool narrow = false;             // (not head) one 4-byte element per lane instead of a 16-byte vector
    long long n = 0;                 // elements every kernel of the run produces
    int gemv() const { return k0 + (pro ? 1 : 0); }
    // per kernel of the run: where its operands come from (a register slot or memory), which slot keeps its
    // output, and whether the output is stored (not if a later kernel of the run overwrites the buffer)
    static constexpr int kMax = pgk::kMergeMaxPhases > pgk::kEpiMaxPhases + 2 ? pgk::kMergeMaxPhases : pgk::kEpiMaxPhases + 2;
    unsigned char src0[kMax] = {}, src1[kMax] = {}, dst[kMax] = {};
    bool store[kMax] = {};
    pgk::Launch launch;
};

struct Segment {
    int k0 = 0, k1 = 0;
    std::vector<MergeGroup> groups;  // cover [k0, k1) in order
    bool has_ext = false;
    int copy_list = -1;             // index into copy_lists
    hipGraph_t g_copy = nullptr, g_ind = nullptr;
    hipGraphExec_t x_copy = nullptr, x_ind = nullptr;
    // host-updated variant: explicit kernel nodes in chain order, two executable instances
    hipGraph_t g_upd = nullptr;
    hipGraphExec_t x_upd[2] = {nullptr, nullptr};
    std::vector<hipGraphNode_t> nodes;
    // indirect graphs of the two table mechanisms that alternate between two instances:
    // [0] PG_TABLE_GRAPH_MEMCPY, [1] PG_TABLE_HOST
    hipGraph_t g_alt[2][2] = {{nullptr, nullptr}, {nullptr, nullptr}};
    hipGraphExec_t x_alt[2][2] = {{nullptr, nullptr}, {nullptr, nullptr}};
};

// A table mechanism whose host-side buffer is read by the GPU when the graph runs, not when the call
// returns: two instances alternate, and an instance is rewritten only after the replay that last
// used it has finished (an event per instance).
struct AltTable {
    bool built = false;
    void* host[2] = {nullptr, nullptr};          // pinned: staging of the in-graph copy, or the table itself
    hipEvent_t ev[2] = {nullptr, nullptr};
    bool used[2] = {false, false};
    unsigned long long cnt = 0;
};

}  // namespace

struct pg_chain {
    std::vector<pg_kernel_desc> k;
    std::vector<pg_tensor_desc> ext, ints, w;
    std::vector<const void*> wptr;
    char* ws = nullptr;
    size_t ws_bytes = 0, ws_need = 0;
    std::vector<size_t> ph_off, int_off;
    std::vector<size_t> shadow_off;     // per internal buffer: its second copy (merged dispatches that rename), or kNoShadow
    size_t table_off = 0;
    std::vector<KernelRec> rec;
    std::vector<Segment> seg;
    std::vector<CopyList> copy_lists;   // [0] = all externals; then one per segment that has any
    std::vector<std::pair<int, int>> eager_fix;   // (kernel, operand) pairs that take a caller pointer
    bool captured = false;
    int device = -1;                    // the device pg_capture ran on (graphs, events and pinned memory belong to it)
    bool eager_only = false;            // built over the static scratch array: pg_eager_static's private chain
    bool merge = true;                  // captured graphs play runs of small kernels with one dispatch
    int table_how = PG_TABLE_KERNARG;
    int copy_how = PG_COPY_KERNEL;
    // host-updated graphs: which instance the next replay rewrites, and when each was last launched
    bool upd_built = false;
    unsigned long long upd_cnt = 0;
    hipEvent_t upd_ev[2] = {nullptr, nullptr};
    bool upd_used[2] = {false, false};
    // pinned staging ring for PG_TABLE_MEMCPY
    static constexpr int kRing = 64;
    void* staging = nullptr;
    size_t staging_stride = 0;
    unsigned long long ring_cnt = 0;
    hipEvent_t ring_ev[2] = {nullptr, nullptr};
    bool ring_used[2] = {false, false};
    AltTable alt[2];                    // [0] PG_TABLE_GRAPH_MEMCPY, [1] PG_TABLE_HOST
};

namespace {

// ---- descriptor validation and layout ------------------------------------------------------------
struct Layout {
    std::vector<size_t> ph_off, int_off, shadow_off;
    size_t table_off = 0;
    std::vector<CopyList> lists;
    std::vector<Segment> seg;
    size_t total = 0;
};

int n_inputs(int op) {
    switch (op) {
    case PG_ADD: case PG_MUL: case PG_RMSNORM: case PG_GEMV: return 2;
    case PG_GELU: return 1;
    case PG_SCALE_BIAS_RELU: return 3;
    default: return -1;
    }
}

bool fits_i32(long long v) { return v > 0 && v <= 0x7fffffffll; }

pg_status validate(const pg_kernel_desc* k, int nk, const pg_tensor_desc* ext, int n_ext,
                   const pg_tensor_desc* ints, int n_int, const pg_tensor_desc* w, int n_w) {
    if (!k || nk <= 0) return fail(PG_EINVAL, "no kernels");
    if (n_ext < 0 || n_int <= 0 || n_w < 0) return fail(PG_EINVAL, "bad tensor counts");
    if ((n_ext && !ext) || !ints || (n_w && !w)) return fail(PG_EINVAL, "null tensor descriptor array");
    auto chk_desc = [&](const pg_tensor_desc* d, int n, const char* what) -> pg_status {
        for (int i = 0; i < n; i++) {
            if (d[i].dtype != PG_F32 && d[i].dtype != PG_BF16) return fail(PG_EINVAL, "%s %d: bad dtype", what, i);
            if (d[i].numel <= 0 || d[i].numel > (1ll << 40)) return fail(PG_EINVAL, "%s %d: bad numel", what, i);
        }
        return PG_OK;
    };
    pg_status st;
    if ((st = chk_desc(ext, n_ext, "ext")) || (st = chk_desc(ints, n_int, "int")) || (st = chk_desc(w, n_w, "weight"))) return st;

    std::vector<long long> written(n_int, 0);   // elements of each internal buffer written so far
    int seg = 0;
    for (int i = 0; i < nk; i++) {
        const pg_kernel_desc& d = k[i];
        const int nin = n_inputs(d.op);
        if (nin < 0) return fail(PG_EINVAL, "kernel %d: bad op %d", i, d.op);
        if (d.dtype != PG_F32 && d.dtype != PG_BF16) return fail(PG_EINVAL, "kernel %d: bad dtype", i);
        if (i == 0 ? d.segment != 0 : (d.segment != seg && d.segment != seg + 1))
            return fail(PG_EINVAL, "kernel %d: segment %d breaks the non-decreasing, gap-free order", i, d.segment);
        seg = d.segment;
        if (d.out.kind != PG_REF_INT || d.out.index < 0 || d.out.index >= n_int)
            return fail(PG_EINVAL, "kernel %d: output must be an internal buffer in range", i);
        if (ints[d.out.index].dtype != d.dtype) return fail(PG_EINVAL, "kernel %d: output dtype mismatch", i);
        long long numel_in[3] = {0, 0, 0};
        for (int j = 0; j < 3; j++) {
            const pg_ref& r = d.in[j];
            if (j >= nin) {
                if (r.kind != PG_REF_NONE) return fail(PG_EINVAL, "kernel %d: operand %d must be unused", i, j);
                continue;
            }
            const pg_tensor_desc* t = nullptr;
            if (r.kind == PG_REF_EXT && r.index >= 0 && r.index < n_ext) t = &ext[r.index];
            else if (r.kind == PG_REF_INT && r.index >= 0 && r.index < n_int) t = &ints[r.index];
            else if (r.kind == PG_REF_WEIGHT && r.index >= 0 && r.index < n_w) t = &w[r.index];
            if (!t) return fail(PG_EINVAL, "kernel %d: operand %d reference out of range", i, j);
            if (t->dtype != d.dtype) return fail(PG_EINVAL, "kernel %d: operand %d dtype mismatch", i, j);
            numel_in[j] = t->numel;
            if (r.kind == PG_REF_INT && r.index == d.out.index) {
                const bool inplace_ok = j == 0 && (d.op == PG_ADD || d.op == PG_MUL || d.op == PG_GELU || d.op == PG_SCALE_BIAS_RELU);
                if (!inplace_ok) return fail(PG_EINVAL, "kernel %d: output overlaps operand %d", i, j);
            }
        }
        long long need[3] = {0, 0, 0}, out_need = 0;
        switch (d.op) {
        case PG_ADD: case PG_MUL: {
            const long long m = d.m ? d.m : d.n;
            if (d.n <= 0 || m <= 0) return fail(PG_EINVAL, "kernel %d: n and m must be positive", i);
            need[0] = d.n; need[1] = m; out_need = d.n;
            break;
        }
        case PG_GELU:
            if (d.n <= 0) return fail(PG_EINVAL, "kernel %d: n must be positive", i);
            need[0] = d.n; out_need = d.n;
            break;
        case PG_RMSNORM:
            if (!fits_i32(d.rows) || !fits_i32(d.cols) || d.n != d.cols) return fail(PG_EINVAL, "kernel %d: bad rows/cols (n must equal cols)", i);
            if (!(d.eps >= 0.f)) return fail(PG_EINVAL, "kernel %d: eps must be >= 0", i);
            need[0] = d.rows * d.cols; need[1] = d.cols; out_need = d.rows * d.cols;
            break;
        case PG_GEMV:
            if (!fits_i32(d.rows) || !fits_i32(d.cols) || !fits_i32(d.n)) return fail(PG_EINVAL, "kernel %d: bad rows/cols/n", i);
            need[0] = d.n * d.cols; need[1] = d.rows * d.cols; out_need = d.rows * d.n;
            break;
        case PG_SCALE_BIAS_RELU: {
            const long long ch = numel_in[1];
            if (d.n <= 0 || d.inner <= 0 || d.inner > 0xffffffffll || ch > 0xffffffffll) return fail(PG_EINVAL, "kernel %d: bad n/inner", i);
            if (numel_in[2] != ch) return fail(PG_EINVAL, "kernel %d: scale and bias sizes differ", i);
            if (ch <= 0 || d.inner > d.n / ch) return fail(PG_EINVAL, "kernel %d: channels*inner exceeds n", i);   // also keeps the product in range
            if (d.n % (ch * d.inner) != 0) return fail(PG_EINVAL, "kernel %d: n is not a multiple of channels*inner", i);
            need[0] = d.n; need[1] = ch; need[2] = ch; out_need = d.n;
            break;
        }
        }
        if (ints[d.out.index].numel < out_need) return fail(PG_EINVAL, "kernel %d: output buffer too small", i);
        for (int j = 0; j < nin; j++) {
            if (numel_in[j] < need[j]) return fail(PG_EINVAL, "kernel %d: operand %d too small", i, j);
            if (d.in[j].kind == PG_REF_INT && written[d.in[j].index] < need[j])
                return fail(PG_EINVAL, "kernel %d: operand %d reads internal buffer %d beyond what earlier kernels wrote", i, j, d.in[j].index);
        }
        written[d.out.index] = std::max(written[d.out.index], out_need);
    }
    return PG_OK;
}

pgk::Shape shape_of(const pg_kernel_desc& d) {
    pgk::Shape sh;
    sh.n = d.n; sh.m = d.m ? d.m : d.n; sh.rows = d.rows; sh.cols = d.cols; sh.inner = d.inner;
    return sh;
}

// Split kernels [k0, k1) of a segment into the runs a captured graph plays with one dispatch each.
// Two kinds of run: a GEMV (the shape k_gemv_shared serves) followed by up to kEpiMaxPhases elementwise
// kernels over its [rows, n] outputs, which become its epilogue -- and preceded, if the kernel before it
// is the RMSNorm that produces its input, by that RMSNorm as a prologue; and up to kMergeMaxPhases
// element-for-element kernels (add / mul / GELU, RMSNorm over rows of one unit) for one workgroup per unit.
// A run grows while the next kernel (a) is of the run's dtype and element count, (b) finds every operand
// that an earlier kernel of the run produced still in a register slot, read element for element (an
// operand produced in the run can never be re-read from memory: its store may not have landed), and
// (c) neither reads with a broadcast period or as an RMSNorm gain a buffer that the run writes, nor
// writes one that the run reads that way, nor (epilogue) writes what the GEMV's other workgroups are
// still reading -- lanes and workgroups of a run work side by side, so only element-for-element reads
// see the right version.  Anything else stands alone.
//
// One exception to (c): every workgroup of a run with a prologue reads all of the RMSNorm's input x,
// and the epilogue may overwrite that very buffer (the residual add of a decoder block does).  Such a run
// renames: it writes the buffer's second copy in the workspace, and the kernels that follow use that copy
// (capture_segment keeps track) -- allowed when the run rewrites the whole buffer.  At the end of a
// segment every buffer must be back in its first copy, where the other modes and the caller look for it:
// a buffer renamed an odd number of times has its last renaming run split back into RMSNorm + GEMV run.
void plan_groups(const pg_kernel_desc* k, int k0, int k1, const pg_tensor_desc* ints, std::vector<MergeGroup>& out) {
    out.clear();
    auto whole = [&](const pg_kernel_desc& d, int j, long long n) {   // operand j is read element for element over all n
        if (d.op == PG_ADD || d.op == PG_MUL) return j == 0 || (d.m ? d.m : d.n) == n;
        return j == 0;                                                  // GELU a, RMSNORM x
    };
    // Is kernel i an RMSNorm [few rows, 2048] straight into a GEMV of the epilogue kernel's shape (its prologue)?
    auto prologue_at = [&](int i) {
        if (!(k[i].op == PG_RMSNORM && k[i].dtype == PG_BF16 && i + 1 < k1 && k[i].rows >= 1 && k[i].rows <= pgk::kPrologueMaxRows)) return false;
        const pg_kernel_desc& v = k[i + 1];
        long long nv = 0;
        if (!(pgk::merge_head(v.op, v.dtype, shape_of(v), &nv) && k[i].cols == v.cols && k[i].rows == v.rows &&
              v.in[1].kind == PG_REF_INT && v.in[1].index == k[i].out.index &&
              !(v.in[0].kind == PG_REF_INT && v.in[0].index == k[i].out.index))) return false;
        // the GEMV itself may overwrite x: renamed like an epilogue kernel's write, if it covers the buffer
        const pg_ref& x = k[i].in[0];
        return !(x.kind == PG_REF_INT && v.out.index == x.index && ints[x.index].numel != nv);
    };
    int i = k0;
    while (i < k1) {
        MergeGroup g;
        g.k0 = i;
        long long n = 0;
        const bool pro = prologue_at(i);
        const int hk = i + (pro ? 1 : 0);
        const bool head = pro || pgk::merge_head(k[i].op, k[i].dtype, shape_of(k[i]), &n);
        if (!head && !pgk::merge_candidate(k[i].op, k[i].dtype, shape_of(k[i]), true, &n)) {
            g.k1 = ++i;
            out.push_back(g);
            continue;
        }
        if (pro) pgk::merge_head(k[hk].op, k[hk].dtype, shape_of(k[hk]), &n);
        g.n = n;
        g.head = head;
        g.pro = pro;
        // a run of small fp32 kernels works one element per lane (no RMSNorm in it); decided by its first kernel
        const bool narrow = !head && k[i].op != PG_RMSNORM && pgk::merge_narrow(k[i].dtype, n);
        g.narrow = narrow;
        int held[pgk::kMergeSlots];                  // internal buffer whose current contents a slot holds, or -1
        for (int& h : held) h = -1;
        std::vector<int> written, broadcast_read;    // internal buffers the run has written / read other than element for element
        int np = 0;
        int h_buf = -1;                              // (epilogue) the internal buffer the GEMV reads h from
        int x_buf = -1;                              // (prologue) the internal buffer the RMSNorm reads
        const int max_phases = head ? pgk::kEpiMaxPhases + 1 + (pro ? 1 : 0) : pgk::kMergeMaxPhases;
        if (head) {
            if (pro) {
                if (k[i].in[0].kind == PG_REF_INT) x_buf = k[i].in[0].index;
                if (k[i].in[1].kind == PG_REF_INT) broadcast_read.push_back(k[i].in[1].index);   // the gain
                written.push_back(k[i].out.index);   // stored by one workgroup, held in no slot: the run cannot read it back
                g.src0[0] = g.src1[0] = (unsigned char)pgk::kMergeFromMemory;
                g.store[0] = true;
                np = 1;
                i++;
            }
            if (k[i].in[1].kind == PG_REF_INT) h_buf = k[i].in[1].index;
            if (k[i].in[0].kind == PG_REF_INT) broadcast_read.push_back(k[i].in[0].index);       // W: every workgroup reads its own rows while others finish
            held[0] = k[i].out.index;
            g.dst[np] = 0;
            g.src0[np] = g.src1[np] = (unsigned char)pgk::kMergeFromMemory;
            written.push_back(k[i].out.index);
            if (k[i].out.index == x_buf) g.rename = x_buf;
            np++;
            i++;
        }
        while (i < k1 && np < max_phases) {
            const pg_kernel_desc& d = k[i];
            long long ni = 0;
            if (!pgk::merge_candidate(d.op, d.dtype, shape_of(d), !head, &ni) || ni != n || d.dtype != k[g.k0].dtype) break;
            if (head && d.op == PG_RMSNORM) break;                       // a row-wide reduction cannot ride in a wave's epilogue
            if (!head && narrow != (d.op != PG_RMSNORM && pgk::merge_narrow(d.dtype, ni))) break;   // one lane width per run
            if (!head && prologue_at(i)) break;                          // left to the GEMV behind it, where it costs next to nothing
            const int nin = n_inputs(d.op);
            unsigned char src[2] = {(unsigned char)pgk::kMergeFromMemory, (unsigned char)pgk::kMergeFromMemory};
            bool ok = true;
            std::vector<int> bc_here;
            for (int j = 0; j < nin && ok; j++) {
                if (d.in[j].kind != PG_REF_INT) continue;
                const int buf = d.in[j].index;
                const bool produced = std::find(written.begin(), written.end(), buf) != written.end();
                if (whole(d, j, n)) {
                    if (!produced) continue;                       // from memory: nothing in the run has touched it yet
                    ok = false;
                    for (int q = 0; q < pgk::kMergeSlots; q++)
                        if (held[q] == buf) { src[j] = (unsigned char)q; ok = true; }
                } else {
                    if (produced) ok = false;
                    bc_here.push_back(buf);
                }
            }
            const int ob = d.out.index;
            if (std::find(broadcast_read.begin(), broadcast_read.end(), ob) != broadcast_read.end() ||
                std::find(bc_here.begin(), bc_here.end(), ob) != bc_here.end() || ob == h_buf) ok = false;
            if (ob == x_buf && ints[ob].numel != n) ok = false;         // would have to rename, and does not rewrite the whole buffer
            if (!ok) break;
            if (ob == x_buf) g.rename = x_buf;
            // slot for the output: the one that holds the buffer's old contents, else a free one, else
            // the one whose buffer the following kernels need last
            int q_out = -1;
            for (int q = 0; q < pgk::kMergeSlots; q++) if (held[q] == ob) q_out = q;
            for (int q = 0; q < pgk::kMergeSlots && q_out < 0; q++) if (held[q] < 0) q_out = q;
            if (q_out < 0) {
                int best_next = -1;
                for (int q = 0; q < pgk::kMergeSlots; q++) {
                    int next = 1 << 30;                                   // never needed again
                    for (int t = i + 1; t < k1 && t < i + 1 + MergeGroup::kMax && next == (1 << 30); t++) {
                        for (int j = 0; j < n_inputs(k[t].op); j++)
                            if (k[t].in[j].kind == PG_REF_INT && k[t].in[j].index == held[q]) next = t;
                        if (k[t].out.index == held[q] && next == (1 << 30)) break;   // overwritten before it is read
                    }
                    if (next > best_next) { best_next = next; q_out = q; }
                }
            }
            held[q_out] = ob;
            g.src0[np] = src[0];
            g.src1[np] = src[1];
            g.dst[np] = (unsigned char)q_out;
            written.push_back(ob);
            broadcast_read.insert(broadcast_read.end(), bc_here.begin(), bc_here.end());
            np++;
            i++;
        }
        if (i == g.k0) i++;      // the first kernel itself was refused (only a descriptor that validation rejects gets here): on its own
        g.k1 = i;
        // an output is stored unless a later kernel of the run overwrites the same buffer (nothing reads memory in between)
        for (int a = 0; a < np; a++) {
            g.store[a] = true;
            for (int t = a + 1; t < np; t++)
                if (k[g.k0 + t].out.index == k[g.k0 + a].out.index) g.store[a] = false;
        }
        if (head && np == 1) g.head = false;         // no prologue, no epilogue: the plain GEMV
        out.push_back(g);
    }
    // every buffer back in its first copy at the end of the segment
    std::vector<int> odd;
    for (const auto& g : out)
        if (g.rename >= 0) {
            auto it = std::find(odd.begin(), odd.end(), g.rename);
            if (it == odd.end()) odd.push_back(g.rename); else odd.erase(it);
        }
    for (int buf : odd) {
        int at = -1;
        for (int gi = 0; gi < (int)out.size(); gi++) if (out[gi].rename == buf) at = gi;
        MergeGroup rms, rest = out[at];
        rms.k0 = rest.k0;
        rms.k1 = rest.k0 + 1;
        rest.k0++;
        rest.pro = false;
        rest.rename = -1;
        for (int t = 0; t + 1 < MergeGroup::kMax; t++) {
            rest.src0[t] = rest.src0[t + 1]; rest.src1[t] = rest.src1[t + 1]; rest.dst[t] = rest.dst[t + 1]; rest.store[t] = rest.store[t + 1];
        }
        if (rest.k1 - rest.k0 == 1) rest.head = false;
        out[at] = rest;
        out.insert(out.begin() + at, rms);
    }
}

void build_copy_list(CopyList& L, const pg_tensor_desc* ext, const std::vector<size_t>& ph_off, char* ws) {
    L.tensors.clear(); L.chunks.clear(); L.groups.clear(); L.bytes = 0;
    for (size_t li = 0; li < L.ext.size(); li++) {
        const int e = L.ext[li];
        const unsigned long long bytes = (unsigned long long)ext[e].numel * elem_bytes(ext[e].dtype);
        L.tensors.push_back({ws ? ws + ph_off[e] : nullptr, bytes});
        L.bytes += (long long)bytes;
    }
    const int nt = (int)L.tensors.size();
    for (int t0 = 0; t0 < nt; t0 += pgk::kCopyMaxSrc) {
        const int t1 = std::min(nt, t0 + pgk::kCopyMaxSrc);
        const int c0 = (int)L.chunks.size();
        for (int t = t0; t < t1; t++)
            for (unsigned long long off = 0; off < L.tensors[t].bytes; off += pgk::kCopyChunkBytes)
                L.chunks.push_back({(unsigned)t, (unsigned)std::min<unsigned long long>(pgk::kCopyChunkBytes, L.tensors[t].bytes - off), off});
        L.groups.push_back({t0, t1, c0, (int)L.chunks.size()});
    }
}

// Lay out the workspace.  ws may be null (size query).  eager_only: the chain will never be captured
// or replayed, so it gets internal buffers only -- no placeholders, pointer table or copy job lists.
void make_layout(const pg_kernel_desc* k, int nk, const pg_tensor_desc* ext, int n_ext,
                 const pg_tensor_desc* ints, int n_int, char* ws, Layout& L, bool eager_only = false) {
    size_t off = 0;
    L.ph_off.assign(n_ext, 0);
    if (!eager_only)
        for (int i = 0; i < n_ext; i++) { L.ph_off[i] = off; off = align_up(off + (size_t)ext[i].numel * elem_bytes(ext[i].dtype)); }
    L.int_off.resize(n_int);
    for (int i = 0; i < n_int; i++) { L.int_off[i] = off; off = align_up(off + (size_t)ints[i].numel * elem_bytes(ints[i].dtype)); }
    L.table_off = off;
    if (!eager_only) off = align_up(off + (size_t)std::max(1, n_ext) * 8);
    // segments and their external sets
    const int n_seg = k[nk - 1].segment + 1;
    L.seg.assign(n_seg, Segment());
    std::vector<std::vector<int>> seg_ext(n_seg);
    for (int i = 0; i < nk; i++) {
        Segment& s = L.seg[k[i].segment];
        if (s.k1 == 0 && (i == 0 || k[i - 1].segment != k[i].segment)) s.k0 = i;
        s.k1 = i + 1;
        for (int j = 0; j < 3; j++)
            if (k[i].in[j].kind == PG_REF_EXT) { s.has_ext = true; seg_ext[k[i].segment].push_back(k[i].in[j].index); }
    }
    L.lists.clear();
    L.lists.emplace_back();
    for (int e = 0; e < n_ext; e++) L.lists[0].ext.push_back(e);
    for (int s = 0; s < n_seg; s++) {
        auto& v = seg_ext[s];
        std::sort(v.begin(), v.end());
        v.erase(std::unique(v.begin(), v.end()), v.end());
        if (v.empty()) continue;
        if ((int)v.size() == n_ext) { L.seg[s].copy_list = 0; continue; }
        L.seg[s].copy_list = (int)L.lists.size();
        L.lists.emplace_back();
        L.lists.back().ext = v;
    }
    if (eager_only) { L.lists.clear(); L.total = off; return; }
    L.shadow_off.assign(n_int, kNoShadow);
    for (auto& sg : L.seg) {
        plan_groups(k, sg.k0, sg.k1, ints, sg.groups);
        for (const auto& g : sg.groups)
            if (g.rename >= 0 && L.shadow_off[g.rename] == kNoShadow) {
                L.shadow_off[g.rename] = off;
                off = align_up(off + (size_t)ints[g.rename].numel * elem_bytes(ints[g.rename].dtype));
            }
    }
    for (auto& cl : L.lists) {
        build_copy_list(cl, ext, L.ph_off, ws);
        cl.tensors_off = off; off = align_up(off + std::max<size_t>(1, cl.tensors.size()) * sizeof(pgk::CopyTensor));
        cl.chunks_off = off; off = align_up(off + std::max<size_t>(1, cl.chunks.size()) * sizeof(pgk::CopyChunk));
    }
    L.total = off;
}

const void* operand_ptr(const pg_chain* c, const pg_ref& r, int mode /*0 eager,1 copy,2 ind*/) {
    switch (r.kind) {
    case PG_REF_WEIGHT: return c->wptr[r.index];
    case PG_REF_INT: return c->ws + c->int_off[r.index];
    case PG_REF_EXT:
        if (c->eager_only) return nullptr;   // no placeholders, no table: the graph forms are never launched
        if (mode == 1) return c->ws + c->ph_off[r.index];
        if (mode == 2) return c->ws + c->table_off + 8 * (size_t)r.index;
        return nullptr;   // patched per call
    default: return nullptr;
    }
}

pg_status make_records(pg_chain* c) {
    const int nk = (int)c->k.size();
    c->rec.assign(nk, KernelRec());
    c->eager_fix.clear();
    for (int i = 0; i < nk; i++) {
        const pg_kernel_desc& d = c->k[i];
        KernelRec& r = c->rec[i];
        r.n_in = n_inputs(d.op);
        for (int j = 0; j < r.n_in; j++)
            if (d.in[j].kind == PG_REF_EXT) { r.ind_mask |= 1 << j; r.ext_of[j] = d.in[j].index; c->eager_fix.push_back({i, j}); }
        ArgBlock* blocks[3] = {&r.a_eager, &r.a_copy, &r.a_ind};
        for (int mode = 0; mode < 3; mode++) {
            ArgBlock& a = *blocks[mode];
            memset(&a, 0, sizeof a);
            a.ptr[0] = c->ws + c->int_off[d.out.index];
            for (int j = 0; j < r.n_in; j++) a.ptr[1 + j] = operand_ptr(c, d.in[j], mode);
            switch (d.op) {
            case PG_ADD: case PG_MUL: case PG_GELU:
                a.ew.n = d.n; a.ew.m = (d.op == PG_GELU) ? d.n : (d.m ? d.m : d.n);
                break;
            case PG_RMSNORM: a.rms.rows = (int)d.rows; a.rms.cols = (int)d.cols; a.rms.eps = d.eps; break;
            case PG_GEMV: a.gemv.rows = (int)d.rows; a.gemv.n = (int)d.n; a.gemv.cols = (int)d.cols; break;
            case PG_SCALE_BIAS_RELU:
                a.sbr.n = d.n; a.sbr.inner = (unsigned)d.inner;
                a.sbr.channels = (unsigned)(d.in[1].kind == PG_REF_EXT ? c->ext[d.in[1].index].numel
                                            : d.in[1].kind == PG_REF_INT ? c->ints[d.in[1].index].numel : c->w[d.in[1].index].numel);
                break;
            }
        }
        const pgk::Shape sh = shape_of(d);
        if (!pgk::plan(d.op, d.dtype, 0, sh, &r.direct) || !pgk::plan(d.op, d.dtype, r.ind_mask, sh, &r.indirect))
            return fail(PG_EINVAL, "kernel %d: no device kernel for op %d dtype %d", i, d.op, d.dtype);
        if (r.direct.grid.x != r.indirect.grid.x || r.direct.block.x != r.indirect.block.x)
            return fail(PG_EINVAL, "kernel %d: direct and indirect forms disagree on the launch shape", i);
        if (d.op == PG_GEMV)
            for (ArgBlock* a : {&r.a_eager, &r.a_copy, &r.a_ind}) a->gemv.row_groups = (int)r.direct.gemm_row_groups;
    }
    for (auto& sg : c->seg)
        for (auto& g : sg.groups) {
            if (g.k1 - g.k0 < 2) continue;
            g.launch = pgk::Launch();
            g.launch.block = dim3(256);
            if (g.head) {
                g.launch.fn = pgk::gemv_epilogue_kernel((int)c->k[g.gemv()].rows, g.pro);
                g.launch.arg_bytes = sizeof(pgk::GemvEpiArgs);
                g.launch.grid = c->rec[g.gemv()].direct.grid;               // the GEMV's own launch shape: same workgroups, same lanes
                if (c->rec[g.gemv()].direct.block.x != 256) return fail(PG_EINVAL, "kernel %d: unexpected GEMV launch shape", g.gemv());
            } else {
                g.launch.fn = pgk::merged_kernel(c->k[g.k0].dtype, g.narrow);
                g.launch.arg_bytes = sizeof(pgk::MergedArgs);
                const long long nvec = g.narrow ? g.n : g.n / (c->k[g.k0].dtype == PG_F32 ? 4 : 8);
                g.launch.grid = dim3((unsigned)((nvec + 255) / 256));       // one workgroup per unit of 256 lanes x 16 bytes
            }
            if (!g.launch.fn) return fail(PG_EINVAL, "kernel %d: no merged kernel for this run", g.k0);
        }
    return PG_OK;
}

// ---- launches ----------------------------------------------------------------------------------------
// The leanest launch the runtime offers: a module function resolved once, the argument block handed
// over as one packed buffer (no per-launch symbol lookup, no per-argument marshalling).
inline hipError_t launch(pgk::Launch& L, void* a, hipStream_t s) {
    if (!L.mod_fn) {
        hipError_t e = hipGetFuncBySymbol(&L.mod_fn, L.fn);
        if (e != hipSuccess) return e;
    }
    size_t sz = L.arg_bytes;
    void* extra[] = {HIP_LAUNCH_PARAM_BUFFER_POINTER, a, HIP_LAUNCH_PARAM_BUFFER_SIZE, &sz, HIP_LAUNCH_PARAM_END};
    return hipModuleLaunchKernel(L.mod_fn, L.grid.x, 1, 1, L.block.x, 1, 1, 0, s, nullptr, extra);
}

pg_status check_call(const pg_chain* c, const void* const* ext, void* stream, bool need_capture) {
    if (!c) return fail(PG_EINVAL, "null chain");
    if (!stream) return fail(PG_EINVAL, "the NULL stream cannot be used; pass a created stream");
    if (need_capture && !c->captured) return fail(PG_ESTATE, "pg_capture has not been called");
    const int n_ext = (int)c->ext.size();
    if (n_ext && !ext) return fail(PG_EINVAL, "null external pointer array");
    for (int i = 0; i < n_ext; i++) {
        if (!ext[i]) return fail(PG_EINVAL, "external pointer %d is null", i);
        if (reinterpret_cast<uintptr_t>(ext[i]) % elem_bytes(c->ext[i].dtype)) return fail(PG_EINVAL, "external pointer %d is not aligned to its element size", i);
    }
    return PG_OK;
}

pg_status run_eager_range(pg_chain* c, int k0, int k1, const void* const* ext, hipStream_t s) {
    for (int i = k0; i < k1; i++) {
        KernelRec& r = c->rec[i];
        for (int j = 0; j < r.n_in; j++)
            if (r.ext_of[j] >= 0) r.a_eager.ptr[1 + j] = ext[r.ext_of[j]];
        PG_HIP(launch(r.direct, &r.a_eager, s));
    }
    return PG_OK;
}

pg_status run_copy_list(pg_chain* c, int list, const void* const* ext, hipStream_t s) {
    CopyList& L = c->copy_lists[list];
    if (c->copy_how == PG_COPY_MEMCPY) {
        for (size_t t = 0; t < L.ext.size(); t++) {
            const int e = L.ext[t];
            PG_HIP(hipMemcpyAsync(c->ws + c->ph_off[e], ext[e], (size_t)c->ext[e].numel * elem_bytes(c->ext[e].dtype),
                                  hipMemcpyDeviceToDevice, s));
        }
        return PG_OK;
    }
    for (const auto& g : L.groups) {
        if (g.c1 == g.c0) continue;
        pgk::CopyArgs a;
        a.chunks = reinterpret_cast<const pgk::CopyChunk*>(c->ws + L.chunks_off) + g.c0;
        a.tensors = reinterpret_cast<const pgk::CopyTensor*>(c->ws + L.tensors_off);
        a.src_base = g.t0;
        a.n_chunks = g.c1 - g.c0;
        for (int t = g.t0; t < g.t1; t++) a.src[t - g.t0] = ext[L.ext[t]];
        void* args[1] = {&a};
        PG_HIP(hipLaunchKernel(pgk::copy_kernel(), dim3((unsigned)a.n_chunks), dim3(256), args, 0, s));
    }
    return PG_OK;
}

pg_status write_table(pg_chain* c, const void* const* ext, hipStream_t s) {
    const int n_ext = (int)c->ext.size();
    if (n_ext == 0) return PG_OK;
    const void** table = reinterpret_cast<const void**>(c->ws + c->table_off);
    if (c->table_how == PG_TABLE_MEMCPY) {
        const int half_len = pg_chain::kRing / 2;
        const int slot = (int)(c->ring_cnt % pg_chain::kRing), half = slot / half_len;
        // the slots of this half were last read by copies issued kRing/2..kRing calls ago: wait for them
        if (slot % half_len == 0 && c->ring_used[half]) PG_HIP(hipEventSynchronize(c->ring_ev[half]));
        char* st = static_cast<char*>(c->staging) + (size_t)slot * c->staging_stride;
        memcpy(st, ext, (size_t)n_ext * 8);
        PG_HIP(hipMemcpyAsync(table, st, (size_t)n_ext * 8, hipMemcpyHostToDevice, s));
        if (slot % half_len == half_len - 1) { PG_HIP(hipEventRecord(c->ring_ev[half], s)); c->ring_used[half] = true; }
        c->ring_cnt++;
        return PG_OK;
    }
    for (int base = 0; base < n_ext; base += pgk::kTableMaxPtrs) {
        pgk::TableArgs a;
        a.table = table;
        a.base = base;
        a.n = std::min(pgk::kTableMaxPtrs, n_ext - base);
        memcpy(a.ptr, ext + base, (size_t)a.n * 8);
        void* args[1] = {&a};
        PG_HIP(hipLaunchKernel(pgk::table_kernel(), dim3(1), dim3(64), args, 0, s));
    }
    return PG_OK;
}

// Before executable graphs, events or pinned staging go away, nothing on the chain's device may still
// use them: a replay may have been issued on another stream than the one at hand, and a copy node of a
// graph reads pinned memory when the graph runs.  Waits for the whole device (graphs are only destroyed
// on the slow path: re-capture and pg_chain_destroy).
void quiesce(pg_chain* c) {
    if (c->device < 0) return;        // never captured: the chain owns no device-side object
    int cur = -1;
    if (hipGetDevice(&cur) != hipSuccess) return;
    if (cur != c->device && hipSetDevice(c->device) != hipSuccess) return;
    (void)hipDeviceSynchronize();
    if (cur != c->device) (void)hipSetDevice(cur);
}

void destroy_update_graphs(pg_chain* c) {
    for (auto& s : c->seg) {
        for (auto& x : s.x_upd) { if (x) (void)hipGraphExecDestroy(x); x = nullptr; }
        if (s.g_upd) (void)hipGraphDestroy(s.g_upd);
        s.g_upd = nullptr;
        s.nodes.clear();
    }
    c->upd_built = false;
    c->upd_used[0] = c->upd_used[1] = false;
}

void destroy_alt_graphs(pg_chain* c) {
    for (auto& s : c->seg)
        for (int v = 0; v < 2; v++)
            for (int i = 0; i < 2; i++) {
                if (s.x_alt[v][i]) (void)hipGraphExecDestroy(s.x_alt[v][i]);
                if (s.g_alt[v][i]) (void)hipGraphDestroy(s.g_alt[v][i]);
                s.x_alt[v][i] = nullptr;
                s.g_alt[v][i] = nullptr;
            }
    for (auto& a : c->alt) { a.built = false; a.used[0] = a.used[1] = false; }
}

void destroy_graphs(pg_chain* c) {
    destroy_update_graphs(c);
    destroy_alt_graphs(c);
    for (auto& s : c->seg) {
        if (s.x_ind && s.x_ind != s.x_copy) (void)hipGraphExecDestroy(s.x_ind);
        if (s.g_ind && s.g_ind != s.g_copy) (void)hipGraphDestroy(s.g_ind);
        if (s.x_copy) (void)hipGraphExecDestroy(s.x_copy);
        if (s.g_copy) (void)hipGraphDestroy(s.g_copy);
        s.x_copy = s.x_ind = nullptr;
        s.g_copy = s.g_ind = nullptr;
    }
    c->captured = false;
}

hipKernelNodeParams node_params(KernelRec& r, void** slot) {
    hipKernelNodeParams p{};
    p.func = const_cast<void*>(r.direct.fn);
    p.gridDim = r.direct.grid;
    p.blockDim = r.direct.block;
    p.sharedMemBytes = 0;
    slot[0] = &r.a_upd;          // every kernel takes its argument block as one by-value struct
    p.kernelParams = slot;
    p.extra = nullptr;
    return p;
}

pg_status build_update_graphs(pg_chain* c, hipStream_t s) {
    if (!c->upd_ev[0]) {
        PG_HIP(hipEventCreateWithFlags(&c->upd_ev[0], hipEventDisableTiming));
        PG_HIP(hipEventCreateWithFlags(&c->upd_ev[1], hipEventDisableTiming));
    }
    for (auto& sg : c->seg) {
        PG_HIP(hipGraphCreate(&sg.g_upd, 0));
        sg.nodes.clear();
        hipGraphNode_t prev = nullptr;
        for (int i = sg.k0; i < sg.k1; i++) {
            KernelRec& r = c->rec[i];
            r.a_upd = r.a_copy;   // external operands start at the placeholders: valid addresses of the right size
            void* slot[1];
            hipKernelNodeParams p = node_params(r, slot);
            hipGraphNode_t n = nullptr;
            PG_HIP(hipGraphAddKernelNode(&n, sg.g_upd, prev ? &prev : nullptr, prev ? 1 : 0, &p));
            sg.nodes.push_back(n);
            prev = n;
        }
        for (auto& x : sg.x_upd) {
            PG_HIP(hipGraphInstantiate(&x, sg.g_upd, nullptr, nullptr, 0));
            PG_HIP(hipGraphUpload(x, s));
        }
    }
    PG_HIP(hipStreamSynchronize(s));
    c->upd_built = true;
    return PG_OK;
}

pg_status run_update(pg_chain* c, const void* const* ext, hipStream_t s) {
    if (!c->upd_built) {
        pg_status st = build_update_graphs(c, s);
        if (st) { destroy_update_graphs(c); return st; }
    }
    const int which = (int)(c->upd_cnt & 1);
    if (c->upd_used[which]) PG_HIP(hipEventSynchronize(c->upd_ev[which]));
    for (auto& sg : c->seg) {
        for (int i = sg.k0; i < sg.k1; i++) {
            KernelRec& r = c->rec[i];
            if (!r.ind_mask) continue;
            for (int j = 0; j < r.n_in; j++)
                if (r.ext_of[j] >= 0) r.a_upd.ptr[1 + j] = ext[r.ext_of[j]];
            void* slot[1];
            hipKernelNodeParams p = node_params(r, slot);
            PG_HIP(hipGraphExecKernelNodeSetParams(sg.x_upd[which], sg.nodes[i - sg.k0], &p));
        }
        PG_HIP(hipGraphLaunch(sg.x_upd[which], s));
    }
    PG_HIP(hipEventRecord(c->upd_ev[which], s));
    c->upd_used[which] = true;
    c->upd_cnt++;
    return PG_OK;
}

// What a captured graph's kernels read their external operands from.
enum GraphKind { kGraphCopy = 0, kGraphTable = 1, kGraphTableMemcpyNode = 2, kGraphHostTable = 3 };

pg_status capture_segment(pg_chain* c, Segment& sg, int kind, int inst, hipStream_t s, hipGraph_t* g_out, hipGraphExec_t* x_out) {
    PG_HIP(hipStreamBeginCapture(s, hipStreamCaptureModeThreadLocal));
    hipError_t le = hipSuccess;
    if (kind == kGraphTableMemcpyNode)   // the graph's first node copies the pointers from its instance's pinned staging
        le = hipMemcpyAsync(c->ws + c->table_off, c->alt[0].host[inst], c->ext.size() * 8, hipMemcpyHostToDevice, s);
    auto block_of = [&](KernelRec& r) -> ArgBlock& { return kind == kGraphCopy ? r.a_copy : kind == kGraphHostTable ? r.a_host[inst] : r.a_ind; };
    // Which copy of each internal buffer is current (see plan_groups: runs that rename).  Every kernel of
    // the segment gets its internal operands in the current copy; all are back in the first at the end.
    std::vector<char> second(c->ints.size(), 0);
    auto in_copy = [&](int buf, bool use_second) -> char* { return c->ws + (use_second ? c->shadow_off[buf] : c->int_off[buf]); };
    auto versioned = [&](int ki, const MergeGroup* grp) -> ArgBlock {     // kernel ki's argument block for this graph
        KernelRec& r = c->rec[ki];
        const pg_kernel_desc& d = c->k[ki];
        ArgBlock a = block_of(r);
        for (int j = 0; j < r.n_in; j++)
            if (d.in[j].kind == PG_REF_INT && second[d.in[j].index]) a.ptr[1 + j] = in_copy(d.in[j].index, true);
        const bool renamed = grp && grp->rename == d.out.index && ki >= grp->gemv();
        if (second[d.out.index] != renamed) a.ptr[0] = in_copy(d.out.index, true);
        return a;
    };
    for (auto& grp : sg.groups) {
        if (le != hipSuccess) break;
        if (!c->merge || grp.k1 - grp.k0 < 2) {
            for (int i = grp.k0; i < grp.k1 && le == hipSuccess; i++) {
                KernelRec& r = c->rec[i];
                ArgBlock a = versioned(i, nullptr);
                le = launch(kind == kGraphCopy ? r.direct : r.indirect, &a, s);
            }
            continue;
        }
        if (grp.head) {
            // the GEMV's dispatch with the following elementwise kernels as its epilogue (and the RMSNorm before it as its prologue)
            pgk::GemvEpiArgs e;
            memset(&e, 0, sizeof e);
            const int hk = grp.gemv();
            KernelRec& hr = c->rec[hk];
            const ArgBlock ha = versioned(hk, &grp);
            e.g = ha.gemv;
            e.head = (kind == kGraphCopy ? 0u : (unsigned)hr.ind_mask) | ((unsigned)grp.dst[hk - grp.k0] << 8) |
                     (grp.store[hk - grp.k0] ? pgk::kEpiHeadStore : 0u);
            if (grp.pro) {
                KernelRec& pr = c->rec[grp.k0];
                const ArgBlock pa = versioned(grp.k0, &grp);
                e.x = pa.ptr[1];
                e.gain = pa.ptr[2];
                e.eps = c->k[grp.k0].eps;
                e.head |= pgk::kEpiPrologue | pgk::kEpiStoreH;
                if (kind != kGraphCopy) e.head |= ((pr.ind_mask & 1) ? pgk::kEpiXSlot : 0u) | ((pr.ind_mask & 2) ? pgk::kEpiGainSlot : 0u);
                // e.g.h is the RMSNorm's output in its current copy: where workgroup 0 stores the normalised rows
            }
            for (int i = hk + 1; i < grp.k1; i++, e.n_epi++) {
                KernelRec& r = c->rec[i];
                const pg_kernel_desc& d = c->k[i];
                const ArgBlock a = versioned(i, &grp);
                const int t = i - grp.k0;
                pgk::MergePhase& ph = e.ph[e.n_epi];
                ph.out = const_cast<void*>(a.ptr[0]);
                ph.in0 = a.ptr[1];
                ph.in1 = r.n_in > 1 ? a.ptr[2] : nullptr;
                ph.m = (d.op == PG_ADD || d.op == PG_MUL) ? (unsigned)(d.m ? d.m : d.n) : (unsigned)grp.n;
                ph.meta = (unsigned)d.op | ((unsigned)grp.src0[t] << 8) | ((unsigned)grp.src1[t] << 16) | ((unsigned)grp.dst[t] << 24);
                ph.ind = (kind == kGraphCopy ? 0u : (unsigned)r.ind_mask) | (grp.store[t] ? pgk::kEpiStore : 0u);
            }
            for (int q = e.n_epi; q < pgk::kEpiMaxPhases; q++) e.ph[q].meta = (unsigned)PG_GELU;   // operands "from slot 0": fetches nothing, never played
            le = launch(grp.launch, &e, s);
            if (grp.rename >= 0) second[grp.rename] ^= 1;
            continue;
        }
        // one dispatch for the run: the kernels' own operands, in order, in one argument struct
        pgk::MergedArgs m;
        memset(&m, 0, sizeof m);
        m.n = (unsigned)grp.n;
        for (int i = grp.k0; i < grp.k1; i++, m.n_phase++) {
            KernelRec& r = c->rec[i];
            const pg_kernel_desc& d = c->k[i];
            const ArgBlock a = versioned(i, nullptr);
            pgk::MergePhase& ph = m.ph[m.n_phase];
            ph.out = const_cast<void*>(a.ptr[0]);
            ph.in0 = a.ptr[1];
            ph.in1 = r.n_in > 1 ? a.ptr[2] : nullptr;
            ph.m = (d.op == PG_ADD || d.op == PG_MUL) ? (unsigned)(d.m ? d.m : d.n) : 0u;
            ph.eps = d.op == PG_RMSNORM ? d.eps : 0.f;
            ph.meta = (unsigned)d.op | ((unsigned)grp.src0[m.n_phase] << 8) | ((unsigned)grp.src1[m.n_phase] << 16) | ((unsigned)grp.dst[m.n_phase] << 24);
            ph.ind = (kind == kGraphCopy ? 0u : (unsigned)r.ind_mask) | (grp.store[m.n_phase] ? pgk::kEpiStore : 0u);
        }
        for (int q = m.n_phase; q < pgk::kMergeMaxPhases; q++) m.ph[q].meta = (unsigned)PG_GELU;   // operands "from slot 0": fetches nothing, never played
        le = launch(grp.launch, &m, s);
    }
    for (char v : second)
        if (v && le == hipSuccess) le = hipErrorAssert;     // plan_groups pairs the renames up; never reached
    hipGraph_t g = nullptr;
    hipError_t ee = hipStreamEndCapture(s, &g);   // always end the capture, even after a failed launch
    if (le != hipSuccess) { if (g) (void)hipGraphDestroy(g); g_hip_err = (int)le; return fail(PG_EHIP, "kernel launch during capture failed: %s", hipGetErrorString(le)); }
    if (ee != hipSuccess) { g_hip_err = (int)ee; return fail(PG_EHIP, "hipStreamEndCapture failed: %s", hipGetErrorString(ee)); }
    hipGraphExec_t x = nullptr;
    hipError_t ie = hipGraphInstantiate(&x, g, nullptr, nullptr, 0);
    if (ie != hipSuccess) { (void)hipGraphDestroy(g); g_hip_err = (int)ie; return fail(PG_EHIP, "hipGraphInstantiate failed: %s", hipGetErrorString(ie)); }
    *g_out = g;
    *x_out = x;
    PG_HIP(hipGraphUpload(x, s));
    return PG_OK;
}

// ---- the indirect refresh of one call, whichever table mechanism is selected ------------------------
struct IndCtx { bool begun = false; int inst = 0; };

pg_status build_alt(pg_chain* c, int v, hipStream_t s) {
    AltTable& a = c->alt[v];
    hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
    PG_HIP(hipStreamIsCapturing(s, &cs));
    if (cs != hipStreamCaptureStatusNone) return fail(PG_EINVAL, "the first indirect replay with this table mechanism builds graphs and cannot run on a capturing stream");
    const size_t bytes = std::max<size_t>(1, c->ext.size()) * 8;
    for (int i = 0; i < 2; i++) {
        if (!a.host[i]) PG_HIP(hipHostMalloc(&a.host[i], bytes, hipHostMallocDefault));
        memset(a.host[i], 0, bytes);
        if (!a.ev[i]) PG_HIP(hipEventCreateWithFlags(&a.ev[i], hipEventDisableTiming));
    }
    if (v == 1)     // kernels dereference slots of the host-resident table: pinned memory has one address on both sides
        for (auto& r : c->rec)
            for (int i = 0; i < 2; i++) {
                r.a_host[i] = r.a_ind;
                for (int j = 0; j < r.n_in; j++)
                    if (r.ext_of[j] >= 0) r.a_host[i].ptr[1 + j] = static_cast<const char*>(a.host[i]) + 8 * (size_t)r.ext_of[j];
            }
    for (auto& sg : c->seg) {
        if (!sg.has_ext) continue;    // such a segment replays its copy graph in every mode
        for (int i = 0; i < 2; i++) {
            pg_status st = capture_segment(c, sg, v == 0 ? kGraphTableMemcpyNode : kGraphHostTable, i, s, &sg.g_alt[v][i], &sg.x_alt[v][i]);
            if (st) { destroy_alt_graphs(c); return st; }
        }
    }
    PG_HIP(hipStreamSynchronize(s));
    a.built = true;
    return PG_OK;
}

pg_status ind_begin(pg_chain* c, const void* const* ext, hipStream_t s, IndCtx& x) {
    if (x.begun) return PG_OK;
    x.begun = true;
    if (c->table_how == PG_TABLE_KERNARG || c->table_how == PG_TABLE_MEMCPY) return write_table(c, ext, s);
    const int v = c->table_how - PG_TABLE_GRAPH_MEMCPY;
    AltTable& a = c->alt[v];
    if (!a.built) { pg_status st = build_alt(c, v, s); if (st) { x.begun = false; return st; } }
    x.inst = (int)(a.cnt & 1);
    if (a.used[x.inst]) PG_HIP(hipEventSynchronize(a.ev[x.inst]));   // the replay that last read this instance
    if (!c->ext.empty()) memcpy(a.host[x.inst], ext, c->ext.size() * 8);
    return PG_OK;
}

hipGraphExec_t ind_exec(pg_chain* c, Segment& sg, const IndCtx& x) {
    if (!sg.has_ext) return sg.x_copy;
    if (c->table_how == PG_TABLE_KERNARG || c->table_how == PG_TABLE_MEMCPY) return sg.x_ind;
    return sg.x_alt[c->table_how - PG_TABLE_GRAPH_MEMCPY][x.inst];
}

pg_status ind_end(pg_chain* c, hipStream_t s, IndCtx& x) {
    if (!x.begun || c->table_how == PG_TABLE_KERNARG || c->table_how == PG_TABLE_MEMCPY) return PG_OK;
    AltTable& a = c->alt[c->table_how - PG_TABLE_GRAPH_MEMCPY];
    PG_HIP(hipEventRecord(a.ev[x.inst], s));
    a.used[x.inst] = true;
    a.cnt++;
    return PG_OK;
}

pg_status run_segment(pg_chain* c, int si, int mode, const void* const* ext, hipStream_t s, IndCtx* ind) {
    Segment& sg = c->seg[si];
    switch (mode) {
    case PG_EAGER: return run_eager_range(c, sg.k0, sg.k1, ext, s);
    case PG_GRAPH_COPY: {
        if (sg.copy_list >= 0) { pg_status st = run_copy_list(c, sg.copy_list, ext, s); if (st) return st; }
        PG_HIP(hipGraphLaunch(sg.x_copy, s));
        return PG_OK;
    }
    case PG_GRAPH_INDIRECT: {
        if (!sg.has_ext) return fail(PG_EUNAVAIL, "segment %d reads no external operand: indirect mode does not exist for it", si);
        pg_status st = ind_begin(c, ext, s, *ind);
        if (st) return st;
        PG_HIP(hipGraphLaunch(ind_exec(c, sg, *ind), s));
        return PG_OK;
    }
    default: return fail(PG_EINVAL, "bad mode %d for segment %d", mode, si);
    }
}

// pg_chain_build, and (eager_only) the private chain pg_eager_static lays over the static scratch array
pg_status build_chain(const pg_kernel_desc* kernels, int32_t nk, const pg_tensor_desc* ext, int32_t n_ext,
                      const pg_tensor_desc* ints, int32_t n_int, const void* const* weight_dev_ptrs,
                      const pg_tensor_desc* weights, int32_t n_w, void* workspace_dev, size_t workspace_bytes,
                      bool eager_only, pg_chain** out) {
    if (!out) return fail(PG_EINVAL, "null out");
    *out = nullptr;
    pg_status st = validate(kernels, nk, ext, n_ext, ints, n_int, weights, n_w);
    if (st) return st;
    if (n_w && !weight_dev_ptrs) return fail(PG_EINVAL, "null weight pointer array");
    for (int i = 0; i < n_w; i++) {
        if (!weight_dev_ptrs[i]) return fail(PG_EINVAL, "weight pointer %d is null", i);
        if (reinterpret_cast<uintptr_t>(weight_dev_ptrs[i]) & 15u) return fail(PG_EINVAL, "weight pointer %d is not 16-byte aligned", i);
    }
    if (!workspace_dev) return fail(PG_EINVAL, "null workspace");
    if (reinterpret_cast<uintptr_t>(workspace_dev) % kAlign) return fail(PG_EINVAL, "workspace is not 256-byte aligned");
    pg_chain* c = new (std::nothrow) pg_chain();
    if (!c) return fail(PG_ENOMEM, "out of host memory");
    c->eager_only = eager_only;
    c->k.assign(kernels, kernels + nk);
    if (n_ext) c->ext.assign(ext, ext + n_ext);
    c->ints.assign(ints, ints + n_int);
    if (n_w) { c->w.assign(weights, weights + n_w); c->wptr.assign(weight_dev_ptrs, weight_dev_ptrs + n_w); }
    c->ws = static_cast<char*>(workspace_dev);
    c->ws_bytes = workspace_bytes;
    Layout L;
    make_layout(c->k.data(), nk, c->ext.data(), n_ext, c->ints.data(), n_int, c->ws, L, eager_only);
    c->ws_need = L.total;
    if (workspace_bytes < L.total) {
        delete c;
        return eager_only ? fail(PG_ENOMEM, "the chain's internal buffers need %zu bytes, the static scratch array holds %zu", L.total, workspace_bytes)
                          : fail(PG_ENOMEM, "workspace has %zu bytes, the chain needs %zu", workspace_bytes, L.total);
    }
    c->ph_off = std::move(L.ph_off);
    c->int_off = std::move(L.int_off);
    c->shadow_off = std::move(L.shadow_off);
    c->table_off = L.table_off;
    c->copy_lists = std::move(L.lists);
    c->seg = std::move(L.seg);
    st = make_records(c);
    if (st) { delete c; return st; }
    *out = c;
    return PG_OK;
}

// ---- pg_eager_static: internal buffers in a static device array ----------------------------------------
// The array's name is a host-side stand-in, not a device address: host code uses only the address
// hipGetSymbolAddress returned for the current device (each GPU holds its own copy at its own address).
static __device__ __align__(256) unsigned char scratch[PG_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
struct StaticSlot {
    void* ptr = nullptr;                 // this device's copy of `scratch`
    pg_chain* chain = nullptr;           // the chain last laid over it (host object only)
    std::vector<unsigned char> key;      // the bytes of the descriptor that chain was built from
};
StaticSlot g_static[kMaxDevices];
std::mutex g_static_mu;

template <typename T>
void key_append(std::vector<unsigned char>& key, const T* p, size_t n) {
    const unsigned char* b = reinterpret_cast<const unsigned char*>(p);
    const unsigned long long count = n;
    key.insert(key.end(), reinterpret_cast<const unsigned char*>(&count), reinterpret_cast<const unsigned char*>(&count) + sizeof count);
    if (n) key.insert(key.end(), b, b + n * sizeof(T));
}

double now_us() {
    return std::chrono::duration<double, std::micro>(std::chrono::steady_clock::now().time_since_epoch()).count();
}

}  // namespace

// ======================================================================================================
extern "C" {

const char* pg_last_error(void) { return g_err.c_str(); }
int pg_last_hip_error(void) { return g_hip_err; }
const char* pg_version(void) { return "pygraph_hip 0.1 (gfx950)"; }

pg_status pg_chain_workspace_bytes(const pg_kernel_desc* kernels, int32_t nk, const pg_tensor_desc* ext, int32_t n_ext,
                                   const pg_tensor_desc* ints, int32_t n_int, size_t* bytes_out) {
    if (!bytes_out) return fail(PG_EINVAL, "null bytes_out");
    // weights are not needed for the layout: only what the layout reads is checked here, pg_chain_build checks the rest
    if (!kernels || nk <= 0) return fail(PG_EINVAL, "no kernels");
    if (n_ext < 0 || n_int <= 0 || (n_ext && !ext) || !ints) return fail(PG_EINVAL, "bad tensor descriptor arrays");
    for (int i = 0; i < nk; i++) {
        if (n_inputs(kernels[i].op) < 0) return fail(PG_EINVAL, "kernel %d: bad op", i);
        if (i == 0 ? kernels[i].segment != 0 : (kernels[i].segment != kernels[i - 1].segment && kernels[i].segment != kernels[i - 1].segment + 1))
            return fail(PG_EINVAL, "kernel %d: bad segment order", i);
        if (kernels[i].out.kind != PG_REF_INT || kernels[i].out.index < 0 || kernels[i].out.index >= n_int)
            return fail(PG_EINVAL, "kernel %d: output must be an internal buffer in range", i);
        for (int j = 0; j < 3; j++) {
            if (kernels[i].in[j].kind == PG_REF_EXT && (kernels[i].in[j].index < 0 || kernels[i].in[j].index >= n_ext))
                return fail(PG_EINVAL, "kernel %d: external reference out of range", i);
            if (kernels[i].in[j].kind == PG_REF_INT && (kernels[i].in[j].index < 0 || kernels[i].in[j].index >= n_int))
                return fail(PG_EINVAL, "kernel %d: internal reference out of range", i);
        }
    }
    for (int i = 0; i < n_ext; i++) if (ext[i].numel <= 0 || ext[i].numel > (1ll << 40) || (ext[i].dtype != PG_F32 && ext[i].dtype != PG_BF16)) return fail(PG_EINVAL, "ext %d: bad descriptor", i);
    for (int i = 0; i < n_int; i++) if (ints[i].numel <= 0 || ints[i].numel > (1ll << 40) || (ints[i].dtype != PG_F32 && ints[i].dtype != PG_BF16)) return fail(PG_EINVAL, "int %d: bad descriptor", i);
    Layout L;
    make_layout(kernels, nk, ext, n_ext, ints, n_int, nullptr, L);
    *bytes_out = L.total;
    return PG_OK;
}

pg_status pg_chain_build(const pg_kernel_desc* kernels, int32_t nk, const pg_tensor_desc* ext, int32_t n_ext,
                         const pg_tensor_desc* ints, int32_t n_int, const void* const* weight_dev_ptrs,
                         const pg_tensor_desc* weights, int32_t n_w, void* workspace_dev, size_t workspace_bytes,
                         pg_chain** out) {
    return build_chain(kernels, nk, ext, n_ext, ints, n_int, weight_dev_ptrs, weights, n_w, workspace_dev, workspace_bytes, false, out);
}

pg_status pg_capture(pg_chain* c, void* hip_stream) {
    if (!c) return fail(PG_EINVAL, "null chain");
    if (!hip_stream) return fail(PG_EINVAL, "capture needs a created stream, not the NULL stream");
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
    PG_HIP(hipStreamIsCapturing(s, &cs));
    if (cs != hipStreamCaptureStatusNone) return fail(PG_EINVAL, "the stream is already capturing");
    quiesce(c);                       // a replay of the old graphs may still be running, on this stream or another
    PG_HIP(hipGetDevice(&c->device));
    destroy_graphs(c);
    // static side of the copy kernel's job lists
    for (auto& L : c->copy_lists) {
        if (!L.tensors.empty()) PG_HIP(hipMemcpyAsync(c->ws + L.tensors_off, L.tensors.data(), L.tensors.size() * sizeof(pgk::CopyTensor), hipMemcpyHostToDevice, s));
        if (!L.chunks.empty()) PG_HIP(hipMemcpyAsync(c->ws + L.chunks_off, L.chunks.data(), L.chunks.size() * sizeof(pgk::CopyChunk), hipMemcpyHostToDevice, s));
    }
    PG_HIP(hipMemsetAsync(c->ws + c->table_off, 0, std::max<size_t>(1, c->ext.size()) * 8, s));
    PG_HIP(hipStreamSynchronize(s));   // the host vectors above may now change; nothing is pending during capture
    if (!c->staging && !c->ext.empty()) {
        c->staging_stride = align_up(c->ext.size() * 8);
        PG_HIP(hipHostMalloc(&c->staging, c->staging_stride * pg_chain::kRing, hipHostMallocDefault));
    }
    for (auto& e : c->ring_ev)
        if (!e && !c->ext.empty()) PG_HIP(hipEventCreateWithFlags(&e, hipEventDisableTiming));
    for (auto& sg : c->seg) {
        pg_status st = capture_segment(c, sg, kGraphCopy, 0, s, &sg.g_copy, &sg.x_copy);
        if (st) { destroy_graphs(c); return st; }
        if (sg.has_ext) {
            st = capture_segment(c, sg, kGraphTable, 0, s, &sg.g_ind, &sg.x_ind);
            if (st) { destroy_graphs(c); return st; }
        } else {
            sg.g_ind = sg.g_copy;   // no external operand: the two graphs would be identical
            sg.x_ind = sg.x_copy;
        }
    }
    PG_HIP(hipStreamSynchronize(s));
    c->captured = true;
    return PG_OK;
}

pg_status pg_eager(pg_chain* c, const void* const* ext, void* hip_stream) {
    pg_status st = check_call(c, ext, hip_stream, false);
    if (st) return st;
    return run_eager_range(c, 0, (int)c->k.size(), ext, static_cast<hipStream_t>(hip_stream));
}

pg_status pg_eager_range(pg_chain* c, const void* const* ext, int32_t k0, int32_t k1, void* hip_stream) {
    pg_status st = check_call(c, ext, hip_stream, false);
    if (st) return st;
    if (k0 < 0 || k1 < k0 || k1 > (int)c->k.size()) return fail(PG_EINVAL, "bad kernel range [%d, %d)", k0, k1);
    return run_eager_range(c, k0, k1, ext, static_cast<hipStream_t>(hip_stream));
}

pg_status pg_eager_static(const pg_kernel_desc* kernels, int32_t nk, const pg_tensor_desc* ext, int32_t n_ext,
                          const pg_tensor_desc* ints, int32_t n_int, const void* const* weight_dev_ptrs,
                          const pg_tensor_desc* weights, int32_t n_w, const void* const* ext_dev_ptrs,
                          int32_t out_int_index, void* out_dev, size_t out_bytes, void* hip_stream) {
    if (!hip_stream) return fail(PG_EINVAL, "the NULL stream cannot be used; pass a created stream");
    if (!out_dev || out_bytes == 0) return fail(PG_EINVAL, "null or empty output buffer");
    if (!kernels || nk <= 0 || n_ext < 0 || n_int <= 0 || n_w < 0 || (n_ext && !ext) || !ints || (n_w && (!weights || !weight_dev_ptrs)))
        return fail(PG_EINVAL, "bad descriptor arrays");
    int dev = -1;
    PG_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(PG_EINVAL, "device ordinal %d out of range", dev);
    std::lock_guard<std::mutex> lock(g_static_mu);
    StaticSlot& slot = g_static[dev];
    if (!slot.ptr) {
        void* p = nullptr;
        PG_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(PG_EHIP, "hipGetSymbolAddress returned a null address for the scratch array");
        slot.ptr = p;
    }
    std::vector<unsigned char> key;
    key_append(key, kernels, (size_t)nk);
    key_append(key, ext, (size_t)n_ext);
    key_append(key, ints, (size_t)n_int);
    key_append(key, weights, (size_t)n_w);
    key_append(key, weight_dev_ptrs, (size_t)n_w);
    if (!slot.chain || key != slot.key) {
        // a new chain: the host-side records are rebuilt (no device memory is touched, nothing is allocated on the device)
        delete slot.chain;
        slot.chain = nullptr;
        slot.key.clear();
        pg_chain* c = nullptr;
        pg_status st = build_chain(kernels, nk, ext, n_ext, ints, n_int, weight_dev_ptrs, weights, n_w, slot.ptr,
                                   (size_t)PG_STATIC_SCRATCH_BYTES, true, &c);
        if (st) return st;
        slot.chain = c;
        slot.key = std::move(key);
    }
    pg_chain* c = slot.chain;
    pg_status st = check_call(c, ext_dev_ptrs, hip_stream, false);
    if (st) return st;
    if (out_int_index < 0 || out_int_index >= n_int) return fail(PG_EINVAL, "bad output buffer index %d", out_int_index);
    const size_t have = (size_t)c->ints[out_int_index].numel * elem_bytes(c->ints[out_int_index].dtype);
    if (out_bytes > have) return fail(PG_EINVAL, "output asks for %zu bytes, internal buffer %d holds %zu", out_bytes, out_int_index, have);
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    // Nothing in the array has to start at zero: pg_chain_build's rule that every read of an internal
    // buffer lies inside what an earlier kernel of the same pass wrote holds here too, so whatever the
    // previous call left behind is overwritten before it can be read.
    if ((st = run_eager_range(c, 0, nk, ext_dev_ptrs, s))) return st;
    PG_HIP(hipMemcpyAsync(out_dev, c->ws + c->int_off[out_int_index], out_bytes, hipMemcpyDeviceToDevice, s));
    return PG_OK;
}

pg_status pg_refresh_copy(pg_chain* c, const void* const* ext, void* hip_stream) {
    pg_status st = check_call(c, ext, hip_stream, true);
    if (st) return st;
    return run_copy_list(c, 0, ext, static_cast<hipStream_t>(hip_stream));
}

pg_status pg_refresh_indirect(pg_chain* c, const void* const* ext, void* hip_stream) {
    pg_status st = check_call(c, ext, hip_stream, true);
    if (st) return st;
    IndCtx x;
    if ((st = ind_begin(c, ext, static_cast<hipStream_t>(hip_stream), x))) return st;
    return ind_end(c, static_cast<hipStream_t>(hip_stream), x);
}

pg_status pg_replay_copy(pg_chain* c, const void* const* ext, void* hip_stream) {
    pg_status st = check_call(c, ext, hip_stream, true);
    if (st) return st;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if ((st = run_copy_list(c, 0, ext, s))) return st;
    for (auto& sg : c->seg) PG_HIP(hipGraphLaunch(sg.x_copy, s));
    return PG_OK;
}

pg_status pg_replay_indirect(pg_chain* c, const void* const* ext, void* hip_stream) {
    pg_status st = check_call(c, ext, hip_stream, true);
    if (st) return st;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    IndCtx x;
    if ((st = ind_begin(c, ext, s, x))) return st;
    for (auto& sg : c->seg) PG_HIP(hipGraphLaunch(ind_exec(c, sg, x), s));
    return ind_end(c, s, x);
}

pg_status pg_replay_update(pg_chain* c, const void* const* ext, void* hip_stream) {
    pg_status st = check_call(c, ext, hip_stream, true);
    if (st) return st;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (!c->upd_built) {
        hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
        PG_HIP(hipStreamIsCapturing(s, &cs));
        if (cs != hipStreamCaptureStatusNone) return fail(PG_EINVAL, "the first pg_replay_update builds graphs and cannot run on a capturing stream");
    }
    return run_update(c, ext, s);
}

pg_status pg_run_selected(pg_chain* c, const uint8_t* mode, const void* const* ext, void* hip_stream) {
    pg_status st = check_call(c, ext, hip_stream, true);
    if (st) return st;
    if (!mode) return fail(PG_EINVAL, "null mode array");
    IndCtx x;
    for (int si = 0; si < (int)c->seg.size(); si++)
        if ((st = run_segment(c, si, mode[si], ext, static_cast<hipStream_t>(hip_stream), &x))) return st;
    return ind_end(c, static_cast<hipStream_t>(hip_stream), x);
}

pg_status pg_select(const double* cost, int32_t n_seg, uint8_t* mode_out) {
    if (!cost || !mode_out || n_seg <= 0) return fail(PG_EINVAL, "bad arguments");
    for (int s = 0; s < n_seg; s++) {
        int best = -1;
        for (int m = 0; m < 3; m++) {
            const double v = cost[3 * s + m];
            if (!std::isfinite(v)) continue;
            if (v < 0) return fail(PG_EINVAL, "segment %d: negative cost", s);
            if (best < 0 || v < cost[3 * s + best]) best = m;
        }
        if (best < 0) return fail(PG_EINVAL, "segment %d has no available variant", s);
        mode_out[s] = (uint8_t)best;
    }
    return PG_OK;
}

pg_status pg_profile(pg_chain* c, const void* const* ext, void* hip_stream, int32_t iters, int32_t inner, double* cost) {
    pg_status st = check_call(c, ext, hip_stream, true);
    if (st) return st;
    if (iters <= 0 || inner <= 0 || !cost) return fail(PG_EINVAL, "bad iters/inner/cost");
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    // one full pass so that every internal buffer holds this iteration's data
    if ((st = run_eager_range(c, 0, (int)c->k.size(), ext, s))) return st;
    PG_HIP(hipStreamSynchronize(s));
    std::vector<double> samples(iters);
    for (int si = 0; si < (int)c->seg.size(); si++) {
        for (int m = 0; m < 3; m++) {
            if (m == PG_GRAPH_INDIRECT && !c->seg[si].has_ext) { cost[3 * si + m] = NAN; continue; }
            for (int it = -2; it < iters; it++) {   // two warm-ups
                const double t0 = now_us();
                for (int r = 0; r < inner; r++) {
                    IndCtx x;
                    if ((st = run_segment(c, si, m, ext, s, &x))) return st;
                    if ((st = ind_end(c, s, x))) return st;
                }
                PG_HIP(hipStreamSynchronize(s));
                if (it >= 0) samples[it] = (now_us() - t0) / inner;
            }
            std::sort(samples.begin(), samples.end());
            cost[3 * si + m] = (iters & 1) ? samples[iters / 2] : 0.5 * (samples[iters / 2 - 1] + samples[iters / 2]);
        }
    }
    return PG_OK;
}

// One whole iteration of a chain in one mode (no per-segment mixture), for the background of pg_profile_in_context.
static pg_status run_whole(pg_chain* c, int mode, const void* const* ext, void* hip_stream) {
    switch (mode) {
    case PG_EAGER: return run_eager_range(c, 0, (int)c->k.size(), ext, static_cast<hipStream_t>(hip_stream));
    case PG_GRAPH_COPY: return pg_replay_copy(c, ext, hip_stream);
    case PG_GRAPH_INDIRECT: return pg_replay_indirect(c, ext, hip_stream);
    default: return fail(PG_EINVAL, "bad background mode %d", mode);
    }
}

pg_status pg_profile_in_context(pg_chain* c, const void* const* ext, pg_chain* bg, const void* const* bg_ext, int32_t bg_mode,
                                void* hip_stream, int32_t iters, int32_t inner, double* cost) {
    pg_status st = check_call(c, ext, hip_stream, true);
    if (st) return st;
    if ((st = check_call(bg, bg_ext, hip_stream, bg_mode != PG_EAGER))) return st;
    if (iters <= 0 || inner <= 0 || !cost) return fail(PG_EINVAL, "bad iters/inner/cost");
    if (bg == c) return fail(PG_EINVAL, "the background chain must be another chain");
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if ((st = run_eager_range(c, 0, (int)c->k.size(), ext, s))) return st;   // every internal buffer holds this iteration's data
    PG_HIP(hipStreamSynchronize(s));
    std::vector<double> samples(iters);
    auto median = [&]() {
        std::sort(samples.begin(), samples.end());
        return (iters & 1) ? samples[iters / 2] : 0.5 * (samples[iters / 2 - 1] + samples[iters / 2]);
    };
    // the background alone: `inner` iterations back to back, then one synchronisation
    for (int it = -2; it < iters; it++) {
        const double t0 = now_us();
        for (int r = 0; r < inner; r++)
            if ((st = run_whole(bg, bg_mode, bg_ext, hip_stream))) return st;
        PG_HIP(hipStreamSynchronize(s));
        if (it >= 0) samples[it] = (now_us() - t0) / inner;
    }
    const double base = median();
    for (int si = 0; si < (int)c->seg.size(); si++) {
        for (int m = 0; m < 3; m++) {
            if (m == PG_GRAPH_INDIRECT && !c->seg[si].has_ext) { cost[3 * si + m] = NAN; continue; }
            for (int it = -2; it < iters; it++) {
                const double t0 = now_us();
                for (int r = 0; r < inner; r++) {
                    if ((st = run_whole(bg, bg_mode, bg_ext, hip_stream))) return st;
                    IndCtx x;
                    if ((st = run_segment(c, si, m, ext, s, &x))) return st;
                    if ((st = ind_end(c, s, x))) return st;
                }
                PG_HIP(hipStreamSynchronize(s));
                if (it >= 0) samples[it] = (now_us() - t0) / inner;
            }
            cost[3 * si + m] = std::max(0.0, median() - base);
        }
    }
    return PG_OK;
}

pg_status pg_time_loop(pg_chain* c, int32_t mode, const uint8_t* mode_per_segment, const void* const* ext_sets, int32_t n_sets,
                       int32_t iters, void* hip_stream, double* us_out) {
    if (!c || !us_out || n_sets <= 0 || iters <= 0) return fail(PG_EINVAL, "bad arguments");
    const int n_ext = (int)c->ext.size();
    pg_status st;
    for (int i = 0; i < n_sets; i++)
        if ((st = check_call(c, ext_sets + (size_t)i * n_ext, hip_stream, mode != PG_EAGER))) return st;
    if (mode == 3 && !mode_per_segment) return fail(PG_EINVAL, "null mode array");
    if (mode < 0 || mode > 4) return fail(PG_EINVAL, "bad mode");
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    PG_HIP(hipStreamSynchronize(s));
    const double t0 = now_us();
    for (int it = 0; it < iters; it++) {
        const void* const* ext = ext_sets + (size_t)(it % n_sets) * n_ext;
        switch (mode) {
        case PG_EAGER: st = run_eager_range(c, 0, (int)c->k.size(), ext, s); break;
        case PG_GRAPH_COPY: st = pg_replay_copy(c, ext, hip_stream); break;
        case PG_GRAPH_INDIRECT: st = pg_replay_indirect(c, ext, hip_stream); break;
        case 4: st = pg_replay_update(c, ext, hip_stream); break;
        default: st = pg_run_selected(c, mode_per_segment, ext, hip_stream); break;
        }
        if (st) return st;
    }
    PG_HIP(hipStreamSynchronize(s));
    *us_out = (now_us() - t0) / iters;
    return PG_OK;
}

// The same loop with an event after every iteration: the time between consecutive events is one
// iteration's completion-to-completion time on the GPU.  The events add a marker per iteration to the
// stream, so the mean of these is slightly above pg_time_loop's; they are for the distribution.
pg_status pg_time_loop_each(pg_chain* c, int32_t mode, const uint8_t* mode_per_segment, const void* const* ext_sets, int32_t n_sets,
                            int32_t iters, void* hip_stream, float* us_each_out) {
    if (!c || !us_each_out || n_sets <= 0 || iters <= 0) return fail(PG_EINVAL, "bad arguments");
    const int n_ext = (int)c->ext.size();
    pg_status st;
    for (int i = 0; i < n_sets; i++)
        if ((st = check_call(c, ext_sets + (size_t)i * n_ext, hip_stream, mode != PG_EAGER))) return st;
    if (mode == 3 && !mode_per_segment) return fail(PG_EINVAL, "null mode array");
    if (mode < 0 || mode > 4) return fail(PG_EINVAL, "bad mode");
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    std::vector<hipEvent_t> ev(iters + 1, nullptr);
    auto cleanup = [&]() { for (auto e : ev) if (e) (void)hipEventDestroy(e); };
    for (auto& e : ev) {
        hipError_t he = hipEventCreate(&e);
        if (he != hipSuccess) { cleanup(); g_hip_err = (int)he; return fail(PG_EHIP, "hipEventCreate failed: %s", hipGetErrorString(he)); }
    }
    hipError_t he = hipStreamSynchronize(s);
    if (he == hipSuccess) he = hipEventRecord(ev[0], s);
    st = PG_OK;
    for (int it = 0; it < iters && he == hipSuccess && st == PG_OK; it++) {
        const void* const* ext = ext_sets + (size_t)(it % n_sets) * n_ext;
        switch (mode) {
        case PG_EAGER: st = run_eager_range(c, 0, (int)c->k.size(), ext, s); break;
        case PG_GRAPH_COPY: st = pg_replay_copy(c, ext, hip_stream); break;
        case PG_GRAPH_INDIRECT: st = pg_replay_indirect(c, ext, hip_stream); break;
        case 4: st = pg_replay_update(c, ext, hip_stream); break;
        default: st = pg_run_selected(c, mode_per_segment, ext, hip_stream); break;
        }
        if (st == PG_OK) he = hipEventRecord(ev[it + 1], s);
    }
    if (he == hipSuccess) he = hipStreamSynchronize(s);     // also after a failed iteration: nothing stays pending on the events
    for (int it = 0; it < iters && he == hipSuccess && st == PG_OK; it++) {
        float ms = 0.f;
        he = hipEventElapsedTime(&ms, ev[it], ev[it + 1]);
        us_each_out[it] = ms * 1e3f;
    }
    cleanup();
    if (st) return st;
    if (he != hipSuccess) { g_hip_err = (int)he; return fail(PG_EHIP, "timed loop failed: %s", hipGetErrorString(he)); }
    return PG_OK;
}

// Launch with start/stop events that take the kernel's own dispatch timestamps.
static pg_status launch_timed(const void* fn, dim3 grid, dim3 block, void* argblock, hipStream_t s,
                              std::vector<hipEvent_t>& evs) {
    hipEvent_t e0 = nullptr, e1 = nullptr;
    PG_HIP(hipEventCreate(&e0));
    evs.push_back(e0);
    PG_HIP(hipEventCreate(&e1));
    evs.push_back(e1);
    void* args[1] = {argblock};
    PG_HIP(hipExtLaunchKernel(fn, grid, block, args, 0, s, e0, e1, 0));
    return PG_OK;
}

static pg_status collect_timed(std::vector<hipEvent_t>& evs, hipStream_t s, float* dur_us, bool sum_all) {
    pg_status st = PG_OK;
    hipError_t e = hipStreamSynchronize(s);
    if (e != hipSuccess) { g_hip_err = (int)e; st = fail(PG_EHIP, "hipStreamSynchronize failed: %s", hipGetErrorString(e)); }
    if (sum_all && dur_us) *dur_us = 0.f;
    for (size_t i = 0; i + 1 < evs.size() && st == PG_OK; i += 2) {
        float ms = 0.f;
        e = hipEventElapsedTime(&ms, evs[i], evs[i + 1]);
        if (e != hipSuccess) { g_hip_err = (int)e; st = fail(PG_EHIP, "hipEventElapsedTime failed: %s", hipGetErrorString(e)); break; }
        if (sum_all) *dur_us += ms * 1000.f; else dur_us[i / 2] = ms * 1000.f;
    }
    for (hipEvent_t ev : evs) (void)hipEventDestroy(ev);
    evs.clear();
    return st;
}

pg_status pg_time_kernels(pg_chain* c, const void* const* ext, int32_t k0, int32_t k1, void* hip_stream, float* dur_us_out) {
    pg_status st = check_call(c, ext, hip_stream, false);
    if (st) return st;
    if (k0 < 0 || k1 < k0 || k1 > (int)c->k.size() || !dur_us_out) return fail(PG_EINVAL, "bad kernel range or null output");
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    std::vector<hipEvent_t> evs;
    evs.reserve(2 * (size_t)(k1 - k0));
    for (int i = k0; i < k1 && st == PG_OK; i++) {
        KernelRec& r = c->rec[i];
        for (int j = 0; j < r.n_in; j++)
            if (r.ext_of[j] >= 0) r.a_eager.ptr[1 + j] = ext[r.ext_of[j]];
        st = launch_timed(r.direct.fn, r.direct.grid, r.direct.block, &r.a_eager, s, evs);
    }
    pg_status st2 = collect_timed(evs, s, dur_us_out, false);
    return st ? st : st2;
}

pg_status pg_time_refresh_copy(pg_chain* c, const void* const* ext, void* hip_stream, float* dur_us_out) {
    pg_status st = check_call(c, ext, hip_stream, true);
    if (st) return st;
    if (!dur_us_out) return fail(PG_EINVAL, "null output");
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    CopyList& L = c->copy_lists[0];
    std::vector<hipEvent_t> evs;
    for (const auto& g : L.groups) {
        if (g.c1 == g.c0 || st != PG_OK) continue;
        pgk::CopyArgs a;
        a.chunks = reinterpret_cast<const pgk::CopyChunk*>(c->ws + L.chunks_off) + g.c0;
        a.tensors = reinterpret_cast<const pgk::CopyTensor*>(c->ws + L.tensors_off);
        a.src_base = g.t0;
        a.n_chunks = g.c1 - g.c0;
        for (int t = g.t0; t < g.t1; t++) a.src[t - g.t0] = ext[L.ext[t]];
        st = launch_timed(pgk::copy_kernel(), dim3((unsigned)a.n_chunks), dim3(256), &a, s, evs);
    }
    pg_status st2 = collect_timed(evs, s, dur_us_out, true);
    return st ? st : st2;
}

pg_status pg_chain_int_buffer(const pg_chain* c, int32_t i, void** p, size_t* bytes) {
    if (!c || i < 0 || i >= (int)c->ints.size()) return fail(PG_EINVAL, "bad internal buffer index");
    if (p) *p = c->ws + c->int_off[i];
    if (bytes) *bytes = (size_t)c->ints[i].numel * elem_bytes(c->ints[i].dtype);
    return PG_OK;
}

pg_status pg_chain_output(const pg_chain* c, int32_t i, void** p, size_t* bytes) { return pg_chain_int_buffer(c, i, p, bytes); }

pg_status pg_chain_placeholder(const pg_chain* c, int32_t i, void** p, size_t* bytes) {
    if (!c || i < 0 || i >= (int)c->ext.size()) return fail(PG_EINVAL, "bad external index");
    if (p) *p = c->ws + c->ph_off[i];
    if (bytes) *bytes = (size_t)c->ext[i].numel * elem_bytes(c->ext[i].dtype);
    return PG_OK;
}

pg_status pg_chain_pointer_table(const pg_chain* c, void** p, size_t* bytes) {
    if (!c) return fail(PG_EINVAL, "null chain");
    if (p) *p = c->ws + c->table_off;
    if (bytes) *bytes = c->ext.size() * 8;
    return PG_OK;
}

pg_status pg_chain_stats(const pg_chain* c, pg_stats* out) {
    if (!c || !out) return fail(PG_EINVAL, "null argument");
    memset(out, 0, sizeof *out);
    out->n_kernels = (int)c->k.size();
    out->n_segments = (int)c->seg.size();
    out->n_ext = (int)c->ext.size();
    for (const auto& r : c->rec) out->n_ext_reading_kernels += r.ind_mask != 0;
    out->copy_bytes_per_replay = c->copy_lists[0].bytes;
    out->table_bytes_per_replay = 8ll * (long long)c->ext.size();
    out->workspace_bytes = (long long)c->ws_need;
    out->copy_chunks = (int)c->copy_lists[0].chunks.size();
    out->captured = c->captured;
    return PG_OK;
}

pg_status pg_chain_launch_shape(const pg_chain* c, int32_t kernel, uint32_t* workgroups_out, uint32_t* threads_out) {
    if (!c || kernel < 0 || kernel >= (int)c->rec.size()) return fail(PG_EINVAL, "bad kernel index");
    if (workgroups_out) *workgroups_out = c->rec[kernel].direct.grid.x;
    if (threads_out) *threads_out = c->rec[kernel].direct.block.x;
    return PG_OK;
}

pg_status pg_set_table_refresh(pg_chain* c, int32_t how) {
    if (!c || how < PG_TABLE_KERNARG || how > PG_TABLE_HOST) return fail(PG_EINVAL, "bad table refresh kind");
    c->table_how = how;
    return PG_OK;
}

pg_status pg_set_dispatch_merge(pg_chain* c, int32_t on) {
    if (!c) return fail(PG_EINVAL, "null chain");
    c->merge = on != 0;
    return PG_OK;
}

pg_status pg_chain_graph_dispatches(const pg_chain* c, int32_t* merged_out, int32_t* unmerged_out) {
    if (!c) return fail(PG_EINVAL, "null chain");
    int n = 0;
    for (const auto& sg : c->seg) n += (int)sg.groups.size();
    if (merged_out) *merged_out = n;
    if (unmerged_out) *unmerged_out = (int)c->k.size();
    return PG_OK;
}

pg_status pg_set_copy_refresh(pg_chain* c, int32_t how) {
    if (!c || (how != PG_COPY_KERNEL && how != PG_COPY_MEMCPY)) return fail(PG_EINVAL, "bad copy refresh kind");
    c->copy_how = how;
    return PG_OK;
}

void pg_chain_destroy(pg_chain* c) {
    if (!c) return;
    quiesce(c);
    destroy_graphs(c);
    for (auto& a : c->alt)
        for (int i = 0; i < 2; i++) {
            if (a.ev[i]) (void)hipEventDestroy(a.ev[i]);
            if (a.host[i]) (void)hipHostFree(a.host[i]);
        }
    if (c->upd_ev[0]) (void)hipEventDestroy(c->upd_ev[0]);
    if (c->upd_ev[1]) (void)hipEventDestroy(c->upd_ev[1]);
    if (c->ring_ev[0]) (void)hipEventDestroy(c->ring_ev[0]);
    if (c->ring_ev[1]) (void)hipEventDestroy(c->ring_ev[1]);
    if (c->staging) (void)hipHostFree(c->staging);
    delete c;
}

}  // extern "C"
