/* A stand-in for the HIP runtime header with just what csrc/cx_hbm.cpp uses, so that its placement policy and its
 * error paths can run on a CPU against a model of device memory (tests/host/hbm_policy_check.cpp implements these). */
#ifndef FAKE_HIP_RUNTIME_H
#define FAKE_HIP_RUNTIME_H
#include <stddef.h>

typedef enum { hipSuccess = 0, hipErrorOutOfMemory = 2, hipErrorInvalidValue = 1 } hipError_t;
typedef struct FakeHandle *hipMemGenericAllocationHandle_t;
typedef enum { hipMemAllocationTypePinned = 1 } hipMemAllocationType;
typedef enum { hipMemLocationTypeDevice = 1 } hipMemLocationType;
typedef struct { hipMemLocationType type; int id; } hipMemLocation;
typedef struct { hipMemAllocationType type; hipMemLocation location; } hipMemAllocationProp;
typedef enum { hipMemAccessFlagsProtReadWrite = 3 } hipMemAccessFlags;
typedef struct { hipMemLocation location; hipMemAccessFlags flags; } hipMemAccessDesc;

hipError_t hipGetDevice(int *device);
hipError_t hipSetDevice(int device);
hipError_t hipGetLastError(void);
hipError_t hipDeviceSynchronize(void);
hipError_t hipMemGetInfo(size_t *free_bytes, size_t *total_bytes);
hipError_t hipMemCreate(hipMemGenericAllocationHandle_t *handle, size_t size, const hipMemAllocationProp *prop, unsigned long long flags);
hipError_t hipMemRelease(hipMemGenericAllocationHandle_t handle);
hipError_t hipMemAddressReserve(void **ptr, size_t size, size_t alignment, void *addr, unsigned long long flags);
hipError_t hipMemAddressFree(void *ptr, size_t size);
hipError_t hipMemMap(void *ptr, size_t size, size_t offset, hipMemGenericAllocationHandle_t handle, unsigned long long flags);
hipError_t hipMemUnmap(void *ptr, size_t size);
hipError_t hipMemSetAccess(void *ptr, size_t size, const hipMemAccessDesc *desc, size_t count);
#endif
