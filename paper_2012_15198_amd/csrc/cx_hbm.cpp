// Placement of the worker matrices in HBM: cx_hbm_alloc / cx_hbm_free.  Host code only (HIP's
// virtual-memory calls); no kernels.  Not an operation of the Crossover-SGD paper: where a
// matrix lies in physical memory decides how fast the mixing kernels of Sections 3 and 3.3 write
// it on this GPU, and a caller cannot place memory with hipMalloc.
//
// What is known, from measurement: on the machines where it shows, the 288 GiB of an MI355X behave
// as three zones of 96 GiB of physical addresses.  A kernel that writes many rows at once (the
// hierarchical mix writes the eight rows of a group per workgroup, the in-place walk wanders over
// all rows) runs at 67-69 % of the HBM peak into a buffer that lies in the zone of the buffer it
// reads, at 73 % into another zone, and at 77-78 % when each buffer is spread over two or three
// zones -- whatever the virtual addresses are.  In a fresh process hipMalloc hands out physical
// memory in address order, so two buffers allocated one after the other mostly share a zone; on
// other machines of the same kind plain buffers lie well by themselves, and spreading costs nothing.
//
// What this file does about it: it takes the free memory of the device in the order the driver
// hands it out (block chunks separated by fillers that stand for the memory skipped), so that
// the chunks of every block lie evenly over everything that was free, maps each block's chunks to
// one virtual range and gives the fillers back.  No assumption on where the zones are.
#include "cx_mix.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdlib>
#include <map>
#include <mutex>
#include <vector>

namespace {

constexpr size_t kGranule = size_t{2} << 20;     // sizes and addresses are multiples of 2 MiB
constexpr size_t kDefaultPiece = size_t{256} << 20;   // physical piece of a block

// CX_HBM_PIECE_MIB in the environment (an even number of MiB, 2 ... 1024) changes the piece size: for measurements
size_t piece_bytes()
{
    if (const char *v = std::getenv("CX_HBM_PIECE_MIB")) {
        const long mib = std::strtol(v, nullptr, 10);
        if (mib >= 2 && mib <= 1024 && mib % 2 == 0) return static_cast<size_t>(mib) << 20;
    }
    return kDefaultPiece;
}
constexpr size_t kFiller = size_t{1} << 30;      // largest piece of skipped memory
constexpr size_t kHeadroom = size_t{8} << 30;    // left untouched for everybody else while the call runs
constexpr int kMaxBlocks = 64;

struct Live { size_t bytes; int device; };
std::mutex g_mutex;
std::map<void *, Live> g_live;

struct Piece {                // one chunk of one block, in creation order
    double where;             // position inside its block, 0..1
    int block;
    size_t offset, bytes;
    hipMemGenericAllocationHandle_t handle;
    bool created = false, mapped = false;
};

hipMemAllocationProp device_memory(int device)
{
    hipMemAllocationProp prop = {};
    prop.type = hipMemAllocationTypePinned;
    prop.location.type = hipMemLocationTypeDevice;
    prop.location.id = device;
    return prop;
}

}  // namespace

int cx_hbm_alloc(void **ptrs_out, const int64_t *bytes, int32_t count, uint32_t flags)
{
    if (!ptrs_out || !bytes) return CX_ERR_NULL;
    if (count < 1 || count > kMaxBlocks) return CX_ERR_SHAPE;
    if (flags != 0) return CX_ERR_UNSUPPORTED;
    std::vector<size_t> size(count);
    size_t need = 0;
    for (int k = 0; k < count; ++k) {
        if (bytes[k] < 1 || bytes[k] > (int64_t{1} << 40)) return CX_ERR_SHAPE;
        size[k] = (static_cast<size_t>(bytes[k]) + kGranule - 1) / kGranule * kGranule;
        need += size[k];
    }
    for (int k = 0; k < count; ++k) ptrs_out[k] = nullptr;

    std::lock_guard<std::mutex> lock(g_mutex);
    int device = 0;
    size_t free_bytes = 0, total_bytes = 0;
    if (hipGetDevice(&device) != hipSuccess || hipMemGetInfo(&free_bytes, &total_bytes) != hipSuccess) {
        (void)hipGetLastError();
        return CX_ERR_HIP;
    }
    if (need > free_bytes) return CX_ERR_MEMORY;
    const hipMemAllocationProp prop = device_memory(device);

    // the chunks of all blocks, sorted by their position inside their block: created in this
    // order with equal fillers between them, every block's chunks end up evenly over the free memory
    const size_t piece = piece_bytes();
    std::vector<Piece> pieces;
    for (int k = 0; k < count; ++k) {
        const size_t n = (size[k] + piece - 1) / piece;
        for (size_t c = 0; c < n; ++c) {
            Piece p;
            p.where = (static_cast<double>(c) + 0.5) / static_cast<double>(n);
            p.block = k;
            p.offset = c * piece;
            p.bytes = std::min(piece, size[k] - p.offset);
            pieces.push_back(p);
        }
    }
    std::stable_sort(pieces.begin(), pieces.end(), [](const Piece &a, const Piece &b) { return a.where < b.where; });
    const size_t spare = free_bytes > need + kHeadroom ? free_bytes - need - kHeadroom : 0;
    const size_t gap = spare / pieces.size() / kGranule * kGranule;

    std::vector<hipMemGenericAllocationHandle_t> fillers;
    std::vector<void *> base(count, nullptr);
    int status = CX_OK;
    bool fill = gap > 0;
    for (Piece &p : pieces) {
        for (size_t done = 0; fill && done < gap;) {
            const size_t skipped = std::min(kFiller, gap - done);
            hipMemGenericAllocationHandle_t h;
            if (hipMemCreate(&h, skipped, &prop, 0) != hipSuccess) {      // less was free than reported: stop skipping
                (void)hipGetLastError();
                fill = false;
                break;
            }
            fillers.push_back(h);
            done += skipped;
        }
        hipError_t made = hipMemCreate(&p.handle, p.bytes, &prop, 0);
        if (made != hipSuccess && !fillers.empty()) {
            // the fillers took what the piece needs (less was free than reported, or somebody else
            // allocated meanwhile): give them back, place the rest without skipping
            (void)hipGetLastError();
            for (hipMemGenericAllocationHandle_t h : fillers) (void)hipMemRelease(h);
            fillers.clear();
            fill = false;
            made = hipMemCreate(&p.handle, p.bytes, &prop, 0);
        }
        if (made != hipSuccess) {
            (void)hipGetLastError();
            status = CX_ERR_MEMORY;
            break;
        }
        p.created = true;
    }
    for (hipMemGenericAllocationHandle_t h : fillers) (void)hipMemRelease(h);

    if (status == CX_OK) {
        for (int k = 0; k < count && status == CX_OK; ++k)
            if (hipMemAddressReserve(&base[k], size[k], kGranule, nullptr, 0) != hipSuccess) {
                (void)hipGetLastError();
                base[k] = nullptr;
                status = CX_ERR_HIP;
            }
    }
    if (status == CX_OK) {
        for (Piece &p : pieces) {
            if (hipMemMap(static_cast<char *>(base[p.block]) + p.offset, p.bytes, 0, p.handle, 0) != hipSuccess) {
                (void)hipGetLastError();
                status = CX_ERR_HIP;
                break;
            }
            p.mapped = true;
        }
    }
    if (status == CX_OK) {
        hipMemAccessDesc access = {};
        access.location = prop.location;
        access.flags = hipMemAccessFlagsProtReadWrite;
        for (int k = 0; k < count && status == CX_OK; ++k)
            if (hipMemSetAccess(base[k], size[k], &access, 1) != hipSuccess) {
                (void)hipGetLastError();
                status = CX_ERR_HIP;
            }
    }
    // a mapping keeps its physical memory alive, so the handles can go now either way
    if (status != CX_OK)
        for (Piece &p : pieces)
            if (p.mapped) (void)hipMemUnmap(static_cast<char *>(base[p.block]) + p.offset, p.bytes);
    for (Piece &p : pieces)
        if (p.created) (void)hipMemRelease(p.handle);
    if (status != CX_OK) {
        for (int k = 0; k < count; ++k)
            if (base[k]) (void)hipMemAddressFree(base[k], size[k]);
        return status;
    }
    for (int k = 0; k < count; ++k) {
        g_live[base[k]] = Live{size[k], device};
        ptrs_out[k] = base[k];
    }
    return CX_OK;
}

int cx_hbm_free(void *ptr)
{
    if (!ptr) return CX_ERR_NULL;
    std::lock_guard<std::mutex> lock(g_mutex);
    const auto it = g_live.find(ptr);
    if (it == g_live.end()) return CX_ERR_UNSUPPORTED;
    const Live block = it->second;
    int current = 0;
    if (hipGetDevice(&current) != hipSuccess) { (void)hipGetLastError(); return CX_ERR_HIP; }
    int status = CX_OK;
    if (current != block.device && hipSetDevice(block.device) != hipSuccess) { (void)hipGetLastError(); return CX_ERR_HIP; }
    // work that still uses the block must have finished before its pages go away
    if (hipDeviceSynchronize() != hipSuccess) status = CX_ERR_HIP;
    if (hipMemUnmap(ptr, block.bytes) != hipSuccess) status = CX_ERR_HIP;
    if (hipMemAddressFree(ptr, block.bytes) != hipSuccess) status = CX_ERR_HIP;
    if (status != CX_OK) (void)hipGetLastError();
    if (current != block.device) (void)hipSetDevice(current);
    g_live.erase(it);
    return status;
}
