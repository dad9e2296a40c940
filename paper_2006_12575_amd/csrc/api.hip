// Status strings, build information, the one tuning switch and per-device launch attributes.
#include <stdlib.h>
#include <string.h>
#include <mutex>
#include <string>
#include <utility>
#include <vector>
#include "internal.h"

extern "C" const char* lamp_status_string(lamp_status s) {
    switch (s) {
        case LAMP_OK: return "ok";
        case LAMP_ERR_NULL: return "a required pointer is NULL";
        case LAMP_ERR_SHAPE: return "bad or mismatching shape";
        case LAMP_ERR_ALIGN: return "pointer or stride not aligned";
        case LAMP_ERR_DTYPE: return "unknown or mismatching dtype";
        case LAMP_ERR_WORKSPACE: return "workspace missing or too small";
        case LAMP_ERR_UNSUPPORTED: return "unsupported request";
        case LAMP_ERR_HIP: return "HIP runtime error";
    }
    return "unknown status";
}

extern "C" const char* lamp_build_info(void) { return "liblamp 0.1 gfx950"; }

namespace lamp {

// LAMP_TUNE="key=value,key=value,..." is parsed once per process; keys are documented in include/lamp.h.
int tune(const char* key, int dflt) {
    static std::once_flag once;
    static std::vector<std::pair<std::string, int>> kv;
    std::call_once(once, [] {
        const char* e = getenv("LAMP_TUNE");
        if (!e) return;
        std::string t(e);
        size_t p = 0;
        while (p < t.size()) {
            size_t q = t.find(',', p);
            if (q == std::string::npos) q = t.size();
            const std::string item = t.substr(p, q - p);
            const size_t eq = item.find('=');
            if (eq != std::string::npos && eq > 0) kv.emplace_back(item.substr(0, eq), atoi(item.c_str() + eq + 1));
            else if (!item.empty()) kv.emplace_back(item, 1);
            p = q + 1;
        }
    });
    for (const auto& it : kv)
        if (it.first == key) return it.second;
    return dflt;
}

// A kernel's dynamic-LDS limit is a per-device attribute of the function: set it once per (device, kernel).
lamp_status ensure_dyn_lds(const void* fn, int bytes) {
    static std::mutex mu;
    static std::vector<std::pair<int, const void*>> done;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return LAMP_ERR_HIP;
    std::lock_guard<std::mutex> lock(mu);
    for (const auto& d : done)
        if (d.first == dev && d.second == fn) return LAMP_OK;
    if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess) return LAMP_ERR_HIP;
    done.emplace_back(dev, fn);
    return LAMP_OK;
}

}  // namespace lamp
