// LUT files: the re-parameterised tables as an artifact on a storage tier (host code only).
//
// Paper: Sec. 3.3 (after re-parameterization the LUT is offloaded to a storage device), the
// offloading setting of Sec. 4.1 and the remark of Sec. 4.2 that the tables sit on large, scalable
// storage devices (only N*d values per token and layer are ever read from them).  The paper gives
// no file format; this one is the simplest that serves the lookup: a 4096-byte little-endian header
// and the raw table.
//
//   offset  0  char[8]  "MOLELUT\0"
//           8  u32      format version (1)
//          12  u32      header bytes (4096) = offset of the payload
//          16  u32      element type (mole_dtype)
//          20  u32      layout (mole_layout)
//          24  i64      V
//          32  i32      L
//          36  i32      N
//          40  i32      d
//          44  u32      0
//          48  u64      payload bytes = L * V * N * d * element size
//   payload: [L, V, N, d] (layer-major) or [V, L, N, d] (id-major: the rows of all layers of one
//   id are one contiguous block, one read per looked-up id).
//
// Reads of looked-up rows use pread on the file descriptor from a few threads, not the mapping, so
// that the destination can be pinned memory and no page of the mapping has to stay resident.
#include "mole_internal.h"

#include <errno.h>
#include <fcntl.h>
#include <string.h>
#include <sys/mman.h>
#include <sys/stat.h>
#include <unistd.h>

#include <atomic>
#include <chrono>
#include <condition_variable>
#include <functional>
#include <mutex>
#include <new>
#include <thread>
#include <vector>

namespace {

// Reader threads that live as long as the file handle: starting threads per call costs more than the
// reads of a decoding step (a few hundred KiB per id).  Workers spin briefly for the next job before
// they sleep on a condition variable.
class WorkerPool {
public:
    ~WorkerPool()
    {
        {
            std::lock_guard<std::mutex> lk(m_);
            stop_ = true;
            ++generation_;
        }
        cv_.notify_all();
        for (auto &t : threads_)
            t.join();
    }
    // body(index, n) on n workers (the caller is worker 0); returns when all are done
    void run(int n, const std::function<void(int, int)> &body)
    {
        if (n <= 1) {
            body(0, 1);
            return;
        }
        while ((int)threads_.size() < n - 1) {
            const int idx = (int)threads_.size() + 1;
            threads_.emplace_back([this, idx] { loop(idx); });
        }
        {
            std::lock_guard<std::mutex> lk(m_);
            body_ = &body;
            n_ = n;
            pending_.store(n - 1, std::memory_order_relaxed);
            generation_.fetch_add(1, std::memory_order_release);
        }
        cv_.notify_all();
        body(0, n);
        while (pending_.load(std::memory_order_acquire) != 0)
            std::this_thread::yield();
    }

private:
    void loop(int idx)
    {
        uint64_t seen = 0;
        for (;;) {
            // spin for about 50 us, then sleep
            const auto t0 = std::chrono::steady_clock::now();
            while (generation_.load(std::memory_order_acquire) == seen) {
                if (std::chrono::steady_clock::now() - t0 > std::chrono::microseconds(50)) {
                    std::unique_lock<std::mutex> lk(m_);
                    cv_.wait(lk, [&] { return generation_.load(std::memory_order_acquire) != seen; });
                    break;
                }
            }
            const std::function<void(int, int)> *body;
            int n;
            {
                std::lock_guard<std::mutex> lk(m_);
                if (stop_)
                    return;
                seen = generation_.load(std::memory_order_relaxed);
                body = body_;
                n = n_;
            }
            if (idx < n) {
                (*body)(idx, n);
                pending_.fetch_sub(1, std::memory_order_release);
            }
        }
    }
    std::vector<std::thread> threads_;
    std::mutex m_;
    std::condition_variable cv_;
    std::atomic<uint64_t> generation_{0};
    std::atomic<int> pending_{0};
    const std::function<void(int, int)> *body_ = nullptr;
    int n_ = 0;
    bool stop_ = false;
};

}  // namespace

struct mole_lut_file {
    int fd;
    int writable;
    void *map;
    size_t map_bytes;
    mole_lut_desc desc;
    int64_t row_bytes;   // N * d * element size
    std::mutex call_mutex;   // calls that use the pool are serialised per handle
    WorkerPool pool;
};

namespace {
using namespace mole;

constexpr uint32_t HEADER_BYTES = 4096;
constexpr uint32_t FORMAT_VERSION = 1;
const char MAGIC[8] = {'M', 'O', 'L', 'E', 'L', 'U', 'T', '\0'};

struct Header {
    char magic[8];
    uint32_t version, header_bytes, dtype, layout;
    int64_t V;
    int32_t L, N, d;
    uint32_t zero;
    uint64_t payload_bytes;
};
static_assert(sizeof(Header) == 56, "header fields are packed without padding");

mole_status check_desc(const char *who, const mole_lut_desc &c)
{
    if (c.dtype != MOLE_F32 && c.dtype != MOLE_BF16 && c.dtype != MOLE_U8)
        return fail(MOLE_EINVAL, "%s: unknown dtype %d", who, c.dtype);
    if (c.layout != MOLE_LAYOUT_LAYER_MAJOR && c.layout != MOLE_LAYOUT_ID_MAJOR)
        return fail(MOLE_EINVAL, "%s: unknown layout %d", who, c.layout);
    if (c.L < 1 || c.N < 1 || c.d < 1 || c.V < 1)
        return fail(MOLE_EINVAL, "%s: bad size (L=%d, V=%lld, N=%d, d=%d)", who, c.L, (long long)c.V, c.N, c.d);
    // the payload size L * V * N * d * element bytes must be representable: a header whose product wraps
    // around could otherwise pass the comparison with the file size
    uint64_t bytes = (uint64_t)c.L;
    if (__builtin_mul_overflow(bytes, (uint64_t)c.V, &bytes) || __builtin_mul_overflow(bytes, (uint64_t)c.N, &bytes) ||
        __builtin_mul_overflow(bytes, (uint64_t)c.d, &bytes) ||
        __builtin_mul_overflow(bytes, (uint64_t)elem_bytes((mole_dtype)c.dtype), &bytes) || bytes > (uint64_t)1 << 62)
        return fail(MOLE_EINVAL, "%s: table of L=%d x V=%lld x N=%d x d=%d elements is too large to address", who, c.L,
                    (long long)c.V, c.N, c.d);
    return MOLE_OK;
}

uint64_t payload_bytes(const mole_lut_desc &c)
{
    return (uint64_t)c.L * (uint64_t)c.V * (uint64_t)c.N * (uint64_t)c.d * elem_bytes((mole_dtype)c.dtype);
}

// byte offset of row block (l, v) inside the payload
inline uint64_t row_offset(const mole_lut_file *f, int l, int64_t v)
{
    const uint64_t rb = (uint64_t)f->row_bytes;
    return f->desc.layout == MOLE_LAYOUT_ID_MAJOR ? ((uint64_t)v * f->desc.L + l) * rb
                                                  : ((uint64_t)l * f->desc.V + v) * rb;
}

int clamp_threads(int threads, int64_t items)
{
    if (threads < 1)
        threads = 1;
    if (threads > 64)
        threads = 64;
    if ((int64_t)threads > items)
        threads = (int)(items > 0 ? items : 1);
    return threads;
}

bool pread_all(int fd, char *dst, uint64_t bytes, uint64_t off)
{
    while (bytes) {
        const ssize_t got = pread(fd, dst, bytes, (off_t)off);
        if (got < 0 && errno == EINTR)
            continue;
        if (got <= 0)
            return false;
        dst += got;
        off += (uint64_t)got;
        bytes -= (uint64_t)got;
    }
    return true;
}

}  // namespace

extern "C" mole_status mole_lut_file_create(const char *path, const mole_lut_desc *desc, mole_lut_file **file)
{
    clear_error();
    if (!path || !desc || !file)
        return fail(MOLE_EINVAL, "mole_lut_file_create: path, desc and file must not be NULL");
    *file = nullptr;
    if (mole_status st = check_desc("mole_lut_file_create", *desc))
        return st;
    const uint64_t pb = payload_bytes(*desc);
    const int fd = open(path, O_RDWR | O_CREAT | O_TRUNC, 0644);
    if (fd < 0)
        return fail(MOLE_EIO, "mole_lut_file_create: cannot create %s: %s", path, strerror(errno));
    if (ftruncate(fd, (off_t)(HEADER_BYTES + pb)) != 0) {
        const int e = errno;
        close(fd);
        return fail(MOLE_EIO, "mole_lut_file_create: cannot size %s to %llu bytes: %s", path,
                    (unsigned long long)(HEADER_BYTES + pb), strerror(e));
    }
    void *map = mmap(nullptr, HEADER_BYTES + pb, PROT_READ | PROT_WRITE, MAP_SHARED, fd, 0);
    if (map == MAP_FAILED) {
        const int e = errno;
        close(fd);
        return fail(MOLE_EIO, "mole_lut_file_create: cannot map %s: %s", path, strerror(e));
    }
    Header h;
    memset(&h, 0, sizeof h);
    memcpy(h.magic, MAGIC, 8);
    h.version = FORMAT_VERSION;
    h.header_bytes = HEADER_BYTES;
    h.dtype = (uint32_t)desc->dtype;
    h.layout = (uint32_t)desc->layout;
    h.V = desc->V;
    h.L = desc->L;
    h.N = desc->N;
    h.d = desc->d;
    h.payload_bytes = pb;
    memset(map, 0, HEADER_BYTES);
    memcpy(map, &h, sizeof h);
    mole_lut_file *f = new (std::nothrow) mole_lut_file;
    if (!f) {
        munmap(map, HEADER_BYTES + pb);
        close(fd);
        return fail(MOLE_EIO, "mole_lut_file_create: out of host memory");
    }
    f->fd = fd;
    f->writable = 1;
    f->map = map;
    f->map_bytes = HEADER_BYTES + pb;
    f->desc = *desc;
    f->desc.reserved = 0;
    f->row_bytes = (int64_t)desc->N * desc->d * (int64_t)elem_bytes((mole_dtype)desc->dtype);
    *file = f;
    return MOLE_OK;
}

extern "C" mole_status mole_lut_file_open(const char *path, mole_lut_file **file, mole_lut_desc *desc)
{
    clear_error();
    if (!path || !file)
        return fail(MOLE_EINVAL, "mole_lut_file_open: path and file must not be NULL");
    *file = nullptr;
    const int fd = open(path, O_RDONLY);
    if (fd < 0)
        return fail(MOLE_EIO, "mole_lut_file_open: cannot open %s: %s", path, strerror(errno));
    struct stat sb;
    Header h;
    if (fstat(fd, &sb) != 0 || (uint64_t)sb.st_size < HEADER_BYTES || !pread_all(fd, (char *)&h, sizeof h, 0)) {
        close(fd);
        return fail(MOLE_EIO, "mole_lut_file_open: %s is shorter than a header", path);
    }
    mole_lut_desc c;
    c.dtype = (int32_t)h.dtype;
    c.layout = (int32_t)h.layout;
    c.L = h.L;
    c.N = h.N;
    c.d = h.d;
    c.reserved = 0;
    c.V = h.V;
    if (memcmp(h.magic, MAGIC, 8) != 0 || h.version != FORMAT_VERSION || h.header_bytes != HEADER_BYTES) {
        close(fd);
        return fail(MOLE_EINVAL, "mole_lut_file_open: %s is not a version-%u LUT file", path, FORMAT_VERSION);
    }
    if (mole_status st = check_desc("mole_lut_file_open", c)) {
        close(fd);
        return st;
    }
    if (h.payload_bytes != payload_bytes(c) || (uint64_t)sb.st_size < HEADER_BYTES + h.payload_bytes) {
        close(fd);
        return fail(MOLE_EINVAL, "mole_lut_file_open: %s: payload size does not match its header", path);
    }
    void *map = mmap(nullptr, HEADER_BYTES + h.payload_bytes, PROT_READ, MAP_SHARED, fd, 0);
    if (map == MAP_FAILED) {
        const int e = errno;
        close(fd);
        return fail(MOLE_EIO, "mole_lut_file_open: cannot map %s: %s", path, strerror(e));
    }
    mole_lut_file *f = new (std::nothrow) mole_lut_file;
    if (!f) {
        munmap(map, HEADER_BYTES + h.payload_bytes);
        close(fd);
        return fail(MOLE_EIO, "mole_lut_file_open: out of host memory");
    }
    f->fd = fd;
    f->writable = 0;
    f->map = map;
    f->map_bytes = HEADER_BYTES + h.payload_bytes;
    f->desc = c;
    f->row_bytes = (int64_t)c.N * c.d * (int64_t)elem_bytes((mole_dtype)c.dtype);
    if (desc)
        *desc = c;
    *file = f;
    return MOLE_OK;
}

extern "C" void *mole_lut_file_payload(mole_lut_file *file)
{
    return file ? static_cast<char *>(file->map) + HEADER_BYTES : nullptr;
}

extern "C" mole_status mole_lut_file_write_layer(mole_lut_file *file, int layer, const void *src_host, int threads)
{
    clear_error();
    if (!file || !src_host)
        return fail(MOLE_EINVAL, "mole_lut_file_write_layer: file and src_host must not be NULL");
    if (!file->writable)
        return fail(MOLE_EINVAL, "mole_lut_file_write_layer: the file was opened read-only");
    if (layer < 0 || layer >= file->desc.L)
        return fail(MOLE_EINVAL, "mole_lut_file_write_layer: layer %d outside [0, %d)", layer, file->desc.L);
    char *payload = static_cast<char *>(file->map) + HEADER_BYTES;
    const char *src = static_cast<const char *>(src_host);
    const int64_t V = file->desc.V;
    const uint64_t rb = (uint64_t)file->row_bytes;
    std::lock_guard<std::mutex> guard(file->call_mutex);
    file->pool.run(clamp_threads(threads, V), [&](int t, int nt) {
        const int64_t v0 = V * t / nt, v1 = V * (t + 1) / nt;
        if (file->desc.layout == MOLE_LAYOUT_LAYER_MAJOR) {
            memcpy(payload + row_offset(file, layer, v0), src + (uint64_t)v0 * rb, (uint64_t)(v1 - v0) * rb);
        } else {
            for (int64_t v = v0; v < v1; ++v)
                memcpy(payload + row_offset(file, layer, v), src + (uint64_t)v * rb, rb);
        }
    });
    return MOLE_OK;
}

extern "C" mole_status mole_lut_file_read_rows(mole_lut_file *file, const int32_t *ids_host, int n,
                                               void *dst_host, int threads)
{
    clear_error();
    if (!file)
        return fail(MOLE_EINVAL, "mole_lut_file_read_rows: file must not be NULL");
    if (n < 0)
        return fail(MOLE_EINVAL, "mole_lut_file_read_rows: n=%d", n);
    if (n == 0)
        return MOLE_OK;
    if (!ids_host || !dst_host)
        return fail(MOLE_EINVAL, "mole_lut_file_read_rows: ids_host and dst_host must not be NULL");
    for (int i = 0; i < n; ++i)
        if (ids_host[i] < 0 || (int64_t)ids_host[i] >= file->desc.V)
            return fail(MOLE_EINVAL, "mole_lut_file_read_rows: ids_host[%d] = %d outside [0, %lld)", i,
                        ids_host[i], (long long)file->desc.V);
    const int L = file->desc.L;
    const uint64_t rb = (uint64_t)file->row_bytes;
    const bool id_major = file->desc.layout == MOLE_LAYOUT_ID_MAJOR;
    // one read per id (id-major) or per (id, layer); threads take reads round-robin
    const int64_t reads = id_major ? (int64_t)n : (int64_t)n * L;
    std::atomic<int> failed{0};
    char *dst = static_cast<char *>(dst_host);
    std::lock_guard<std::mutex> guard(file->call_mutex);
    file->pool.run(clamp_threads(threads, reads), [&](int t, int nt) {
        for (int64_t r = t; r < reads && !failed.load(std::memory_order_relaxed); r += nt) {
            bool ok;
            if (id_major) {
                ok = pread_all(file->fd, dst + (uint64_t)r * L * rb, (uint64_t)L * rb,
                               HEADER_BYTES + row_offset(file, 0, ids_host[r]));
            } else {
                const int i = (int)(r / L), l = (int)(r % L);
                ok = pread_all(file->fd, dst + ((uint64_t)i * L + l) * rb, rb,
                               HEADER_BYTES + row_offset(file, l, ids_host[i]));
            }
            if (!ok)
                failed.store(1, std::memory_order_relaxed);
        }
    });
    if (failed.load())
        return fail(MOLE_EIO, "mole_lut_file_read_rows: read failed: %s", strerror(errno));
    return MOLE_OK;
}

extern "C" mole_status mole_lut_file_close(mole_lut_file *file)
{
    clear_error();
    if (!file)
        return MOLE_OK;
    mole_status st = MOLE_OK;
    if (file->writable && msync(file->map, file->map_bytes, MS_SYNC) != 0)
        st = fail(MOLE_EIO, "mole_lut_file_close: msync failed: %s", strerror(errno));
    munmap(file->map, file->map_bytes);
    close(file->fd);
    delete file;
    return st;
}
