/*
 * Runs the library's decode path -- host planning and the decode kernels' own source --
 * on host threads (hip/hip_runtime.h and l3_gfx950.h beside this file) and compares what it
 * writes with expected bytes from a case file.  "Device" buffers are heap blocks of exactly
 * the size the interface promises (a file's block ends with the 16-byte granule that holds
 * its last byte), so under AddressSanitizer any access outside them ends the run; under
 * ThreadSanitizer any two accesses to LDS or to the outputs that no barrier orders do.
 *
 * usage: kernel_cpu <case file>       (written by tests/test_kernel_cpu_build.py)
 * With L3CPU_RECORD=<directory> in the environment every decode launch is recorded there
 * (which kernel, grid, argument block, every live buffer with its address and contents) and
 * so are the buffers after the run: what tests/native/isa_interp/interp.py needs to run the
 * same launch from the compiler's machine code.
 * Test infrastructure.
 */
#include <hip/hip_runtime.h>

#include "l3_gfx950.h"

/* the kernel source under test: the library's, unless the build names another (a copy with a
 * planted mistake, to show that the sanitizers see it) */
#ifndef L3_KERNEL_SOURCE
#define L3_KERNEL_SOURCE "../../../paper_2208_08711_amd/csrc/l3_device.hip"
#endif
#include L3_KERNEL_SOURCE

#include <cstdio>
#include <string>

void l3_encode_state_free(L3EncodeState*) {}
void l3_ablation_state_free(L3AblationState*) {}

namespace {

/* what a recorded launch says about its kernel: patch size, mode, how the descriptors travel
 * (0 device table, 1 up to 32 in the arguments, 2 up to 256), and the sizes of its first and
 * last argument (the others are gx, count, status, crop_w, crop_h, top_priority_below, table pointer) */
struct KernelFacts { int n, mode, kind; size_t first_bytes, tail_bytes; };
std::map<const void*, KernelFacts> g_facts;
int g_recorded = 0;

void write_regions(FILE* f) {
    const uint64_t count = l3cpu::regions().size();
    std::fwrite(&count, 8, 1, f);
    for (const auto& r : l3cpu::regions()) {
        const uint64_t address = (uint64_t)(uintptr_t)r.first, bytes = r.second;
        std::fwrite(&address, 8, 1, f);
        std::fwrite(&bytes, 8, 1, f);
        std::fwrite(r.first, 1, r.second, f);
    }
}

void record_launch(const char* dir, const void* kernel, dim3 grid, dim3 block, void** a) {
    const KernelFacts k = g_facts.at(kernel);
    FILE* f = std::fopen((std::string(dir) + "/launch_" + std::to_string(g_recorded++) + ".bin").c_str(), "wb");
    if (!f) std::abort();
    const int32_t head[6] = {k.n, k.mode, k.kind, (int32_t)grid.x, (int32_t)block.x, 0};
    std::fwrite(head, 4, 6, f);
    /* the argument block as the GPU sees it: every argument at its natural alignment */
    std::vector<uint8_t> block_bytes(k.first_bytes + 40 + k.tail_bytes, 0);
    std::memcpy(block_bytes.data(), a[0], k.first_bytes);
    const size_t o = k.first_bytes;
    std::memcpy(&block_bytes[o], a[1], 4);
    std::memcpy(&block_bytes[o + 4], a[2], 4);
    std::memcpy(&block_bytes[o + 8], a[3], 8);
    std::memcpy(&block_bytes[o + 16], a[4], 4);
    std::memcpy(&block_bytes[o + 20], a[5], 4);
    std::memcpy(&block_bytes[o + 24], a[6], 4);
    std::memcpy(&block_bytes[o + 32], a[7], 8);
    std::memcpy(&block_bytes[o + 40], a[8], k.tail_bytes);
    const uint64_t bytes = block_bytes.size();
    std::fwrite(&bytes, 8, 1, f);
    std::fwrite(block_bytes.data(), 1, bytes, f);
    write_regions(f);
    std::fclose(f);
}

template <int N, int MODE>
void register_kernels() {
    typedef typename TailFor<MODE>::type Tail;
    auto& reg = l3cpu::registry();
    g_facts[reinterpret_cast<const void*>(&l3_decode_kernel<N, 4, MODE>)] = {N, MODE, 0, 8, sizeof(Tail)};
    g_facts[reinterpret_cast<const void*>(&l3_decode_kernel_args<N, 4, MODE, kArgDescsSmall>)] =
        {N, MODE, 1, sizeof(DescPack<kArgDescsSmall>), sizeof(Tail)};
    g_facts[reinterpret_cast<const void*>(&l3_decode_kernel_args<N, 4, MODE, kArgDescs>)] =
        {N, MODE, 2, sizeof(DescPack<kArgDescs>), sizeof(Tail)};
    reg[reinterpret_cast<const void*>(&l3_decode_kernel<N, 4, MODE>)] = [](void** a) {
        l3_decode_kernel<N, 4, MODE>(*static_cast<const L3ImageDesc**>(a[0]), *static_cast<uint32_t*>(a[1]),
                                     *static_cast<uint32_t*>(a[2]), *static_cast<uint32_t**>(a[3]),
                                     *static_cast<uint32_t*>(a[4]), *static_cast<uint32_t*>(a[5]),
                                     *static_cast<uint32_t*>(a[6]), *static_cast<const uint16_t**>(a[7]),
                                     *static_cast<Tail*>(a[8]));
    };
    reg[reinterpret_cast<const void*>(&l3_decode_kernel_args<N, 4, MODE, kArgDescsSmall>)] = [](void** a) {
        l3_decode_kernel_args<N, 4, MODE, kArgDescsSmall>(
            *static_cast<DescPack<kArgDescsSmall>*>(a[0]), *static_cast<uint32_t*>(a[1]),
            *static_cast<uint32_t*>(a[2]), *static_cast<uint32_t**>(a[3]), *static_cast<uint32_t*>(a[4]),
            *static_cast<uint32_t*>(a[5]), *static_cast<uint32_t*>(a[6]), *static_cast<const uint16_t**>(a[7]),
            *static_cast<Tail*>(a[8]));
    };
    reg[reinterpret_cast<const void*>(&l3_decode_kernel_args<N, 4, MODE, kArgDescs>)] = [](void** a) {
        l3_decode_kernel_args<N, 4, MODE, kArgDescs>(
            *static_cast<DescPack<kArgDescs>*>(a[0]), *static_cast<uint32_t*>(a[1]),
            *static_cast<uint32_t*>(a[2]), *static_cast<uint32_t**>(a[3]), *static_cast<uint32_t*>(a[4]),
            *static_cast<uint32_t*>(a[5]), *static_cast<uint32_t*>(a[6]), *static_cast<const uint16_t**>(a[7]),
            *static_cast<Tail*>(a[8]));
    };
}
template <int N>
void register_patch_size() {
    register_kernels<N, L3_MODE_HWC>();
    register_kernels<N, L3_MODE_CHW>();
    register_kernels<N, L3_MODE_TENSOR>();
}

struct Reader {
    FILE* f;
    template <class T> T get() {
        T v;
        if (std::fread(&v, sizeof v, 1, f) != 1) { std::fprintf(stderr, "case file too short\n"); std::exit(2); }
        return v;
    }
    std::vector<uint8_t> bytes(size_t n) {
        std::vector<uint8_t> v(n);
        if (n && std::fread(v.data(), 1, n, f) != n) { std::fprintf(stderr, "case file too short\n"); std::exit(2); }
        return v;
    }
};

constexpr uint8_t kPoison = 0xA5;

int fail(const char* what, int image, size_t at) {
    std::fprintf(stderr, "MISMATCH: %s, image %d, byte %zu\n", what, image, at);
    return 1;
}

}  // namespace

int main(int argc, char** argv) {
    if (argc != 2) return 2;
    register_patch_size<32>();
    register_patch_size<64>();
    register_patch_size<128>();
    Reader in{std::fopen(argv[1], "rb")};
    if (!in.f) return 2;
    if (in.get<uint32_t>() != 0x434B334Cu) return 2;   /* "L3KC" */
    const uint32_t mode = in.get<uint32_t>();          /* 0 interleaved, 1 planar, 2 fused, 3 fused through the call that allocates nothing */
    const int n = (int)in.get<uint32_t>();
    const uint32_t crop_w = in.get<uint32_t>(), crop_h = in.get<uint32_t>();
    float mean[3], stdv[3];
    for (float& m : mean) m = in.get<float>();
    for (float& s : stdv) s = in.get<float>();
    const uint32_t dtype = in.get<uint32_t>();
    const uint32_t pad_cols = in.get<uint32_t>();

    std::vector<uint8_t*> blocks, outs;
    std::vector<std::vector<uint8_t>> expected;
    std::vector<l3_item> items((size_t)n);
    std::vector<l3_crop> crops((size_t)n);
    std::vector<size_t> out_bytes((size_t)n, 0);
    for (int i = 0; i < n; ++i) {
        const size_t len = (size_t)in.get<uint64_t>();
        const std::vector<uint8_t> file = in.bytes(len);
        /* the file at an odd place in a block that ends with its last 16-byte granule */
        const size_t shift = (size_t)((i * 7 + 1) % 16);
        const size_t block_len = (shift + len + 15) / 16 * 16;
        uint8_t* block = static_cast<uint8_t*>(std::aligned_alloc(16, block_len));
        std::memset(block, 0xEE, block_len);
        std::memcpy(block + shift, file.data(), len);
        blocks.push_back(block);
        l3_item& it = items[(size_t)i];
        it.d_file = block + shift;
        it.file_len = len;
        if (l3_peek_header(file.data(), len, &it.info) != L3_OK) { std::fprintf(stderr, "bad file %d\n", i); return 2; }
        crops[(size_t)i].x0 = in.get<int32_t>();
        crops[(size_t)i].y0 = in.get<int32_t>();
        crops[(size_t)i].flip = (uint8_t)in.get<uint32_t>();
        const uint32_t w = it.info.width, h = it.info.height;
        if (mode == 0) {
            it.out_row_stride = 3 * (size_t)w + pad_cols;
            out_bytes[(size_t)i] = it.out_row_stride * h;
        } else if (mode == 1) {
            it.out_row_stride = (size_t)w + pad_cols;
            out_bytes[(size_t)i] = it.out_row_stride * h * 3;
        }
        if (mode <= 1) {
            uint8_t* out = static_cast<uint8_t*>(std::malloc(out_bytes[(size_t)i]));
            std::memset(out, kPoison, out_bytes[(size_t)i]);
            outs.push_back(out);
            it.d_out = out;
            expected.push_back(in.bytes((size_t)in.get<uint64_t>()));
        } else {
            it.d_out = nullptr;
            it.out_row_stride = 0;
        }
    }
    std::vector<uint8_t> expected_tensor;
    uint8_t* tensor = nullptr;
    const size_t tensor_bytes = (size_t)n * 3 * crop_w * crop_h * 2;
    if (mode >= 2) {
        expected_tensor = in.bytes((size_t)in.get<uint64_t>());
        if (expected_tensor.size() != tensor_bytes) return 2;
        tensor = static_cast<uint8_t*>(std::malloc(tensor_bytes));
        std::memset(tensor, kPoison, tensor_bytes);
    }
    uint32_t* status = static_cast<uint32_t*>(std::malloc(sizeof(uint32_t) * (size_t)n));
    std::memset(status, 0xFF, sizeof(uint32_t) * (size_t)n);

    const char* record_dir = std::getenv("L3CPU_RECORD");
    if (record_dir) {
        for (size_t i = 0; i < blocks.size(); ++i)
            l3cpu::regions()[blocks[i]] = ((i * 7 + 1) % 16 + items[i].file_len + 15) / 16 * 16;
        for (size_t i = 0; i < outs.size(); ++i) l3cpu::regions()[outs[i]] = out_bytes[i];
        if (tensor) l3cpu::regions()[tensor] = tensor_bytes;
        l3cpu::regions()[status] = sizeof(uint32_t) * (size_t)n;
        l3cpu::launch_observer() = [record_dir](const void* kernel, dim3 grid, dim3 block, void** a) {
            record_launch(record_dir, kernel, grid, block, a);
        };
    }
    l3_ctx* ctx = nullptr;
    if (l3_ctx_create(&ctx, 0) != L3_OK) return 2;
    l3_status st;
    if (mode <= 1)
        st = l3_decode_batch(ctx, items.data(), n, mode == 0 ? L3_LAYOUT_HWC : L3_LAYOUT_CHW, status, nullptr);
    else if (mode == 2)
        st = l3_decode_crop_normalize_batch(ctx, items.data(), crops.data(), n, crop_w, crop_h, mean, stdv,
                                            (l3_dtype)dtype, tensor, status, nullptr);
    else
        st = l3_decode_crop_normalize_batch_noalloc(ctx, items.data(), crops.data(), n, crop_w, crop_h, mean,
                                                    stdv, (l3_dtype)dtype, tensor, status, nullptr);
    if (st != L3_OK) { std::fprintf(stderr, "call failed: %s\n", l3_status_string(st)); return 1; }
    if (record_dir) {
        FILE* f = std::fopen((std::string(record_dir) + "/after.bin").c_str(), "wb");
        if (!f) std::abort();
        write_regions(f);
        std::fclose(f);
    }
    l3_ctx_destroy(ctx);

    int rc = 0;
    for (int i = 0; i < n && rc == 0; ++i) {
        if (status[i] != 0) rc = fail("status word not zero", i, status[i]);
        if (mode > 1) continue;
        const l3_item& it = items[(size_t)i];
        const uint32_t w = it.info.width, h = it.info.height;
        const size_t row = mode == 0 ? 3 * (size_t)w : w, rows = mode == 0 ? h : 3 * (size_t)h;
        if (expected[(size_t)i].size() != row * rows) return 2;
        for (size_t y = 0; y < rows && rc == 0; ++y)
            for (size_t x = 0; x < it.out_row_stride; ++x) {
                const uint8_t got = outs[(size_t)i][y * it.out_row_stride + x];
                const uint8_t want = x < row ? expected[(size_t)i][y * row + x] : kPoison;
                if (got != want) { rc = fail(x < row ? "pixel" : "wrote between the rows", i, y * it.out_row_stride + x); break; }
            }
    }
    if (mode >= 2 && rc == 0)
        for (size_t k = 0; k < tensor_bytes; ++k)
            if (tensor[k] != expected_tensor[k]) { rc = fail("tensor", (int)(k / (tensor_bytes / (size_t)n)), k); break; }
    for (uint8_t* b : blocks) std::free(b);
    for (uint8_t* o : outs) std::free(o);
    std::free(tensor);
    std::free(status);
    std::fclose(in.f);
    if (rc == 0) std::printf("ok: %d images, mode %u\n", n, mode);
    return rc;
}
