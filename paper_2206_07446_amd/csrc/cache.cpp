// On-disk cache of post-transformation weights (Section 3.1.2): the decision stage stores
// the transformed weights of the kernels it picked, the cold start reads them back instead of
// running the weight transformation.  Host code only: file I/O, a pinned staging ring and
// asynchronous copies to the device.
#include <fcntl.h>
#include <sys/stat.h>
#include <unistd.h>
#include <cerrno>
#include <chrono>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <vector>
#include "nnv_internal.h"

using namespace nnv;

namespace {

constexpr size_t kHeaderBlock = 4096;         // the payload starts at this file offset (O_DIRECT alignment)
constexpr size_t kPiece = 8u << 20;           // bytes per read / copy
constexpr uint32_t kFormat = 1;
const char kMagic[8] = {'N', 'N', 'V', 'C', 'A', 'C', 'H', 'E'};

struct Header {
    char magic[8];
    uint32_t format, layout_version, kind, dtype;
    int32_t k, c, r, s, groups;
    uint32_t reserved;
    uint64_t payload_bytes;
    uint64_t checksum;
};
static_assert(sizeof(Header) <= kHeaderBlock, "header must fit its block");

// Order-dependent 64-bit checksum over 8-byte words (the tail is zero-extended).
struct Checksum {
    uint64_t h = 0x9E3779B97F4A7C15ull;
    void add(const void *p, size_t n) {
        const unsigned char *b = static_cast<const unsigned char *>(p);
        size_t i = 0;
        for (; i + 8 <= n; i += 8) {
            uint64_t w;
            memcpy(&w, b + i, 8);
            h = ((h << 7) | (h >> 57)) ^ w;
            h *= 0xD6E8FEB86659FD93ull;
        }
        if (i < n) {
            uint64_t w = 0;
            memcpy(&w, b + i, n - i);
            h = ((h << 7) | (h >> 57)) ^ w;
            h *= 0xD6E8FEB86659FD93ull;
        }
    }
};

Header make_header(const nnv_conv_desc *d, int kind, uint64_t bytes) {
    Header h;
    memset(&h, 0, sizeof h);
    memcpy(h.magic, kMagic, 8);
    h.format = kFormat;
    h.layout_version = (uint32_t)nnv_layout_version();
    h.kind = (uint32_t)kind;
    h.dtype = kind == NNV_DIRECT ? (uint32_t)NNV_F32 : (uint32_t)d->dtype;   // raw weights are always float32
    h.k = d->k; h.c = d->c; h.r = d->r; h.s = d->s; h.groups = d->groups;
    h.payload_bytes = bytes;
    return h;
}

bool same_layer(const Header &a, const Header &b) {
    return memcmp(a.magic, b.magic, 8) == 0 && a.format == b.format && a.layout_version == b.layout_version &&
           a.kind == b.kind && a.dtype == b.dtype && a.k == b.k && a.c == b.c && a.r == b.r && a.s == b.s &&
           a.groups == b.groups && a.payload_bytes == b.payload_bytes;
}

int check_args(const char *path, const nnv_conv_desc *desc, nnv_kind kind, const void *w_tx, size_t *bytes) {
    if (!path || !desc || !w_tx) return NNV_E_NULL;
    if (kind < 0 || kind >= NNV_KIND_COUNT) return NNV_E_ARG;
    const int sup = nnv_kind_supported(desc, kind);
    if (sup < 0) return sup;
    if (sup == 0) return NNV_E_UNSUPPORTED;
    *bytes = nnv_transformed_bytes(desc, kind);
    return *bytes ? NNV_OK : NNV_E_UNSUPPORTED;
}

bool write_all(int fd, const void *p, size_t n) {
    const char *b = static_cast<const char *>(p);
    while (n) {
        const ssize_t w = write(fd, b, n);
        if (w < 0) {
            if (errno == EINTR) continue;
            return false;
        }
        b += w;
        n -= (size_t)w;
    }
    return true;
}

// Reads exactly n bytes at `off` unless the file ends first; returns the bytes read or -1.
ssize_t pread_full(int fd, void *p, size_t n, off_t off) {
    char *b = static_cast<char *>(p);
    size_t got = 0;
    while (got < n) {
        const ssize_t r = pread(fd, b + got, n - got, off + (off_t)got);
        if (r < 0) {
            if (errno == EINTR) continue;
            return -1;
        }
        if (r == 0) break;
        got += (size_t)r;
    }
    return (ssize_t)got;
}

// Two pinned pieces, allocated once per process on first use and never freed.
std::mutex g_lock;
char *g_stage[2] = {nullptr, nullptr};
hipEvent_t g_done[2];

hipError_t ensure_stage() {
    if (g_stage[0]) return hipSuccess;
    void *p = nullptr;
    hipError_t e = hipHostMalloc(&p, 2 * kPiece, hipHostMallocDefault);
    if (e != hipSuccess) return e;
    for (int i = 0; i < 2; ++i) {
        e = hipEventCreateWithFlags(&g_done[i], hipEventDisableTiming);
        if (e != hipSuccess) return e;
    }
    g_stage[0] = static_cast<char *>(p);
    g_stage[1] = g_stage[0] + kPiece;
    return hipSuccess;
}

double ms_since(std::chrono::steady_clock::time_point t0) {
    return std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count();
}

}  // namespace

extern "C" {

int nnv_cache_write(const char *path, const nnv_conv_desc *desc, nnv_kind kind, const void *w_tx, void *hip_stream) {
    size_t bytes = 0;
    int rc = check_args(path, desc, kind, w_tx, &bytes);
    if (rc) return rc;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    hipError_t e = hipStreamSynchronize(st);
    if (e != hipSuccess) return record_hip_error(e);
    std::vector<char> host(bytes);
    e = hipMemcpy(host.data(), w_tx, bytes, hipMemcpyDeviceToHost);
    if (e != hipSuccess) return record_hip_error(e);
    Checksum cs;
    cs.add(host.data(), bytes);
    std::vector<char> block(kHeaderBlock, 0);
    Header h = make_header(desc, kind, bytes);
    h.checksum = cs.h;
    memcpy(block.data(), &h, sizeof h);
    const int fd = open(path, O_WRONLY | O_CREAT | O_TRUNC, 0644);
    if (fd < 0) return NNV_E_IO;
    const bool ok = write_all(fd, block.data(), block.size()) && write_all(fd, host.data(), bytes) && fsync(fd) == 0;
    const int saved = errno;
    close(fd);
    errno = saved;
    return ok ? NNV_OK : NNV_E_IO;
}

int nnv_cache_read(const char *path, const nnv_conv_desc *desc, nnv_kind kind, void *w_tx, int verify, void *hip_stream,
                   nnv_cache_io *io) {
    size_t bytes = 0;
    int rc = check_args(path, desc, kind, w_tx, &bytes);
    if (rc) return rc;
    if (reinterpret_cast<uintptr_t>(w_tx) & 15) return NNV_E_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const auto t0 = std::chrono::steady_clock::now();
    int direct = 1;
    int fd = open(path, O_RDONLY | O_DIRECT);
    if (fd < 0 && errno == EINVAL) {      // file system without O_DIRECT
        direct = 0;
        fd = open(path, O_RDONLY);
    }
    if (fd < 0) return NNV_E_IO;
    if (!direct) (void)posix_fadvise(fd, 0, 0, POSIX_FADV_DONTNEED);

    double file_ms = 0.0;
    auto timed_read = [&](void *dst, size_t n, off_t off) {
        const auto t = std::chrono::steady_clock::now();
        const ssize_t r = pread_full(fd, dst, n, off);
        file_ms += ms_since(t);
        return r;
    };
    auto fail = [&](int code) {
        const int saved = errno;
        close(fd);
        errno = saved;
        return code;
    };

    // header block (checked before anything touches the device or w_tx)
    alignas(4096) static thread_local char head[kHeaderBlock];
    ssize_t got = timed_read(head, kHeaderBlock, 0);
    if (got < 0) return fail(NNV_E_IO);
    if ((size_t)got < kHeaderBlock) return fail(NNV_E_CACHE);
    Header h;
    memcpy(&h, head, sizeof h);
    if (!same_layer(h, make_header(desc, kind, bytes))) return fail(NNV_E_CACHE);
    struct stat sb;
    if (fstat(fd, &sb) != 0) return fail(NNV_E_IO);
    if ((uint64_t)sb.st_size < kHeaderBlock + bytes) return fail(NNV_E_CACHE);

    std::lock_guard<std::mutex> guard(g_lock);
    hipError_t e = ensure_stage();
    if (e != hipSuccess) { fail(NNV_E_HIP); return record_hip_error(e); }

    // payload: read piece i into buffer i % 2 once the copy that last used it has finished
    Checksum cs;
    const size_t pieces = (bytes + kPiece - 1) / kPiece;
    bool used[2] = {false, false};
    for (size_t i = 0; i < pieces; ++i) {
        const int b = (int)(i & 1);
        const size_t off = i * kPiece;
        const size_t n = bytes - off < kPiece ? bytes - off : kPiece;
        if (used[b]) {
            e = hipEventSynchronize(g_done[b]);
            if (e != hipSuccess) { fail(NNV_E_HIP); return record_hip_error(e); }
        }
        // O_DIRECT wants whole 4096-byte blocks: round the request up, a short read at the end of the file is fine
        const size_t ask = direct ? (n + kHeaderBlock - 1) / kHeaderBlock * kHeaderBlock : n;
        got = timed_read(g_stage[b], ask, (off_t)(kHeaderBlock + off));
        if (got < 0 && direct && errno == EFAULT) {
            // this kernel cannot DMA file blocks straight into pinned device-visible memory:
            // go on with buffered reads (the file's cached pages dropped first)
            close(fd);
            fd = open(path, O_RDONLY);
            if (fd < 0) return NNV_E_IO;
            direct = 0;
            (void)posix_fadvise(fd, 0, 0, POSIX_FADV_DONTNEED);
            got = timed_read(g_stage[b], n, (off_t)(kHeaderBlock + off));
        }
        if (got < 0) return fail(NNV_E_IO);
        if ((size_t)got < n) return fail(NNV_E_CACHE);
        if (verify) cs.add(g_stage[b], n);
        e = hipMemcpyAsync(static_cast<char *>(w_tx) + off, g_stage[b], n, hipMemcpyHostToDevice, st);
        if (e == hipSuccess) e = hipEventRecord(g_done[b], st);
        if (e != hipSuccess) { fail(NNV_E_HIP); return record_hip_error(e); }
        used[b] = true;
    }
    e = hipStreamSynchronize(st);
    close(fd);
    if (e != hipSuccess) return record_hip_error(e);
    if (io) {
        io->total_ms = ms_since(t0);
        io->file_ms = file_ms;
        io->bytes = (double)bytes;
        io->direct_io = direct;
    }
    if (verify && cs.h != h.checksum) return NNV_E_CACHE;
    return NNV_OK;
}

}  // extern "C"
