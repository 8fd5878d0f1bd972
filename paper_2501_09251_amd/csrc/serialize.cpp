// Plans on disk.  The paper amortises its preprocessing over iterative use (Section 4.3.2); a
// saved plan extends that across processes: the row reordering of a large graph takes seconds
// to tens of seconds, reading the plan back takes as long as the file.
//
// Layout: a fixed header (magic, format version, the sizes of the option and statistics structs
// as a compatibility check), the option and statistics structs, the scalar fields of the plan,
// then every array as a 64-bit element count followed by its bytes, in the order of `visit`,
// then a 64-bit checksum of everything before it.  The kernels index memory by what the arrays
// hold, so a file whose contents changed after it was written must not reach them: the loader
// refuses it.  Byte order and struct layout are those of the machine that wrote the file.
#include <cstdio>
#include <cstring>
#include <string>

#include "internal.h"

namespace accspmm {
namespace {

constexpr char kMagic[8] = {'A', 'C', 'C', 'S', 'P', 'M', 'M', '\n'};
constexpr uint32_t kFormatVersion = 1;

struct Header {
    char magic[8];
    uint32_t version, options_size, stats_size, reserved;
};

struct Scalars {
    int32_t WH, TW, NW, n_hot;
    int64_t M, W, T, nnz, sum_dw, n_slots;
};

// Four interleaved multiply-xor lanes over 64-bit words (one dependent chain would run at a
// fraction of the disk rate on a 2 GB plan); both sides feed it the same sequence of pieces.
class Checksum {
public:
    void update(const void* p, size_t n) {
        const unsigned char* b = static_cast<const unsigned char*>(p);
        for (; n >= 32; n -= 32, b += 32) {
            uint64_t w[4];
            std::memcpy(w, b, 32);
            for (int k = 0; k < 4; ++k) lane_[k] = (lane_[k] ^ w[k]) * kMul + 1;
        }
        for (; n; --n, ++b) lane_[0] = (lane_[0] ^ *b) * kMul + 1;
    }
    uint64_t value() const {
        uint64_t h = 0;
        for (int k = 0; k < 4; ++k) h = (h ^ lane_[k] ^ (lane_[k] >> 29)) * kMul;
        return h ^ (h >> 32);
    }

private:
    static constexpr uint64_t kMul = 0x9e3779b97f4a7c15ull;
    uint64_t lane_[4] = {1, 2, 3, 4};
};

class Writer {
public:
    explicit Writer(const char* path) : f_(std::fopen(path, "wb")) {
        if (!f_) fail(ACC_SPMM_ERR_INVALID_ARG, std::string("cannot open ") + path + " for writing");
    }
    ~Writer() { if (f_) std::fclose(f_); }
    void bytes(const void* p, size_t n) {
        if (n && std::fwrite(p, 1, n, f_) != n) fail(ACC_SPMM_ERR_INVALID_ARG, "write failed (disk full?)");
        sum_.update(p, n);
    }
    template <class T> void host(const std::vector<T>& v) {
        const uint64_t n = v.size();
        bytes(&n, sizeof n);
        bytes(v.data(), n * sizeof(T));
    }
    template <class T> void device(const DevBuf<T>& b) {
        std::vector<T> tmp(b.n);
        if (b.n) ACC_HIP(hipMemcpy(tmp.data(), b.p, b.n * sizeof(T), hipMemcpyDeviceToHost));
        host(tmp);
    }
    void close() {
        const uint64_t sum = sum_.value();
        bytes(&sum, sizeof sum);
        const int rc = std::fclose(f_);
        f_ = nullptr;
        if (rc != 0) fail(ACC_SPMM_ERR_INVALID_ARG, "write failed on close");
    }

private:
    std::FILE* f_;
    Checksum sum_;
};

class Reader {
public:
    explicit Reader(const char* path) : f_(std::fopen(path, "rb")) {
        if (!f_) fail(ACC_SPMM_ERR_INVALID_ARG, std::string("cannot open ") + path);
        std::fseek(f_, 0, SEEK_END);
        size_ = (uint64_t)std::ftell(f_);
        std::fseek(f_, 0, SEEK_SET);
    }
    ~Reader() { std::fclose(f_); }
    void bytes(void* p, size_t n) {
        if (n && std::fread(p, 1, n, f_) != n) fail(ACC_SPMM_ERR_INVALID_ARG, "plan file is truncated");
        sum_.update(p, n);
    }
    template <class T> void host(std::vector<T>& v) {
        uint64_t n = 0;
        bytes(&n, sizeof n);
        if (n > size_ / sizeof(T)) fail(ACC_SPMM_ERR_INVALID_ARG, "plan file is corrupt (array longer than the file)");
        v.resize(n);
        bytes(v.data(), n * sizeof(T));
    }
    template <class T> void device(DevBuf<T>& b) {
        std::vector<T> tmp;
        host(tmp);
        b.upload(tmp.data(), tmp.size());
    }
    // the stored checksum follows everything read so far and ends the file
    void close() {
        const uint64_t expected = sum_.value();
        uint64_t stored = 0;
        bytes(&stored, sizeof stored);
        if (stored != expected) fail(ACC_SPMM_ERR_INVALID_ARG, "plan file is corrupt (checksum mismatch)");
        if (std::fgetc(f_) != EOF) fail(ACC_SPMM_ERR_INVALID_ARG, "plan file is corrupt (bytes after the checksum)");
    }

private:
    std::FILE* f_;
    uint64_t size_ = 0;
    Checksum sum_;
};

// the arrays of a plan, in file order; A is a Writer or a Reader
template <class A, class P>
void visit(A& a, P& plan) {
    a.host(plan.perm);
    a.host(plan.iperm);
    a.host(plan.parent);
    a.host(plan.col_order);
    a.host(plan.col_rank);
    a.host(plan.items);
    a.host(plan.splits);
    a.device(plan.fmt.row_window_offset);
    a.device(plan.fmt.tc_offset);
    a.device(plan.fmt.sparse_a_to_b);
    a.device(plan.fmt.tc_local_bit);
    a.device(plan.fmt.vals);
    a.device(plan.d_perm_pad);
    a.device(plan.a2b_plain);
    a.device(plan.d_entry_of);
    a.device(plan.d_rowptr);
    a.device(plan.d_colidx);
    a.device(plan.d_vals);
}

}  // namespace

void save_plan(const Plan& plan, const char* path) {
    if (!path) fail(ACC_SPMM_ERR_INVALID_ARG, "null path");
    int dev = -1;
    ACC_HIP(hipGetDevice(&dev));
    if (dev != plan.device) fail(ACC_SPMM_ERR_INVALID_ARG, "the plan lives on another device than the current one");
    Writer w(path);
    Header h{};
    std::memcpy(h.magic, kMagic, sizeof kMagic);
    h.version = kFormatVersion;
    h.options_size = (uint32_t)sizeof(acc_spmm_options);
    h.stats_size = (uint32_t)sizeof(acc_spmm_stats);
    w.bytes(&h, sizeof h);
    w.bytes(&plan.opt, sizeof plan.opt);
    w.bytes(&plan.stats, sizeof plan.stats);
    const DeviceFormat& f = plan.fmt;
    const Scalars s{f.WH, f.TW, f.NW, plan.n_hot, f.M, f.W, f.T, f.nnz, f.sum_dw, plan.n_slots};
    w.bytes(&s, sizeof s);
    visit(w, plan);
    w.close();
}

acc_spmm_plan_t* load_plan(const char* path) {
    if (!path) fail(ACC_SPMM_ERR_INVALID_ARG, "null path");
    Reader r(path);
    Header h{};
    r.bytes(&h, sizeof h);
    if (std::memcmp(h.magic, kMagic, sizeof kMagic) != 0) fail(ACC_SPMM_ERR_INVALID_ARG, "not a plan file");
    if (h.version != kFormatVersion || h.options_size != sizeof(acc_spmm_options) || h.stats_size != sizeof(acc_spmm_stats))
        fail(ACC_SPMM_ERR_UNSUPPORTED, "plan file was written by another version of the library");
    int dev_count = 0;
    if (hipGetDeviceCount(&dev_count) != hipSuccess || dev_count == 0)
        fail(ACC_SPMM_ERR_HIP, "no HIP device: this library only runs on a gfx950 GPU (there is no CPU path)");
    acc_spmm_plan_t* handle = new acc_spmm_plan_t;
    Plan& P = handle->plan;
    try {
        ACC_HIP(hipGetDevice(&P.device));
        prepare_static_scratch();
        r.bytes(&P.opt, sizeof P.opt);
        r.bytes(&P.stats, sizeof P.stats);
        Scalars s{};
        r.bytes(&s, sizeof s);
        DeviceFormat& f = P.fmt;
        f.WH = s.WH; f.TW = s.TW; f.NW = s.NW;
        f.M = s.M; f.W = s.W; f.T = s.T; f.nnz = s.nnz; f.sum_dw = s.sum_dw;
        P.n_hot = s.n_hot;
        P.n_slots = s.n_slots;
        visit(r, P);
        r.close();
        // consistency of what the kernels index by
        if (f.M != P.stats.M || (int64_t)P.perm.size() != f.M || (int64_t)f.row_window_offset.n != f.W + 1 ||
            (int64_t)f.tc_offset.n != f.T + 1 || (int64_t)f.sparse_a_to_b.n != f.T * f.TW ||
            (int64_t)f.tc_local_bit.n != f.T * f.NW || (int64_t)f.vals.n < f.nnz || (int64_t)P.d_perm_pad.n != f.W * f.WH)
            fail(ACC_SPMM_ERR_INVALID_ARG, "plan file is corrupt (array sizes do not fit together)");
        P.d_items.upload(P.items.data(), P.items.size());
        P.d_splits.upload(P.splits.data(), P.splits.size());
        if (!P.col_order.empty()) P.d_col_order.upload(P.col_order.data(), P.col_order.size());
    } catch (...) {
        delete handle;
        throw;
    }
    return handle;
}

}  // namespace accspmm
