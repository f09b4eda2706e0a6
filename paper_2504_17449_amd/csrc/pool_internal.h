// What the request queue needs to know about a pool (the pool itself stays opaque).
#pragma once
#include <hip/hip_runtime.h>
#include "../../include/hmi.h"

const hmi_pool_config_t* hmi_internal_config(const hmi_pool_t* pool);
hipStream_t hmi_internal_compute_stream(const hmi_pool_t* pool);
// every layer of the tenant has been registered (hmi_pool_load_tenant / hmi_pool_alias_tenant)
bool hmi_internal_tenant_ready(const hmi_pool_t* pool, int32_t tenant);
