/* What the CPU stand-in of the HIP runtime records about kernel launches (test infrastructure). */
#ifndef DFT3D_HOSTSIM_H
#define DFT3D_HOSTSIM_H
#include <stddef.h>
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif
typedef struct {
    const char* name;    /* demangled kernel name */
    unsigned grid[3], block[3];
    size_t dynamic_lds;
    const void* src;     /* tensor the launch reads, NULL when the kernel's arguments are not decoded */
    void* dst;           /* tensor it writes */
    int64_t src_bytes, dst_bytes;   /* extents from src / dst that the launch may touch */
} hostsim_launch;
size_t hostsim_launch_count(void);
const hostsim_launch* hostsim_launches(void);
void hostsim_clear_log(void);
const char* hostsim_failure(void);   /* first violated check, or NULL */
size_t hostsim_live_allocations(void);
/* "Device" tensors for the driver: an address range of the given size that is registered as a live
 * allocation but has no memory behind it (the host code under test never touches tensor data). */
void* hostsim_reserve(size_t bytes);
void hostsim_release(void* p, size_t bytes);
#ifdef __cplusplus
}
#endif
#endif
